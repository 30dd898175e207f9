// Host launchers of the gradient kernels (bwd_kernels.h), instantiated for the state counts the selective-scan layout
// uses with one lane per chain.
#include "bwd_kernels.h"
#include "launch.h"

namespace bm {

bool bwd_supported(int d_state) { return d_state == 4 || d_state == 8 || d_state == 16; }
int bwd_chunk_tokens(int d_state, bool dense)
{
    if (dense) return d_state <= 4 ? kBwdChunk<4, true> : d_state <= 8 ? kBwdChunk<8, true> : kBwdChunk<16, true>;
    return d_state <= 4 ? kBwdChunk<4, false> : d_state <= 8 ? kBwdChunk<8, false> : kBwdChunk<16, false>;
}

// The dense form (two waves per SIMD) once the walk has more waves than the chip has SIMDs; see kBwdChunk.
bool bwd_dense(int d_inner, int batch) { return 2LL * ((d_inner + 63) / 64) * batch > 4LL * cu_count(); }

// Zeroes a float buffer (the accumulation targets of the atomics above); a kernel rather than a memset node so that
// the call can be captured into a graph.
__global__ __launch_bounds__(256) void bwd_zero_kernel(float* p, long long n)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

__global__ __launch_bounds__(256) void bwd_bc_kernel(const BwdBcArgs a)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const int two_n = 2 * a.N;
    if (i >= a.rows * two_n) return;
    const long long r = i / two_n;
    const int v = (int)(i % two_n);
    const float* src = a.part + r * a.slots * two_n + v;
    float acc = 0.0f;
    for (int k = 0; k < a.slots; k++) acc += src[(long long)k * two_n];
    if (v < a.N) a.dB[r * a.N + v] = acc;
    else a.dC[r * a.N + v - a.N] = acc;
}

void launch_bwd_bc(const BwdBcArgs& a, hipStream_t st)
{
    const long long n = a.rows * 2 * a.N;
    if (n <= 0) return;
    hipLaunchKernelGGL(bwd_bc_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
}

template <int N, typename IO, bool DENSE>
static void launch_pair(const BwdArgs& a, int batch, hipStream_t st)
{
    const dim3 grid((unsigned)(((a.Dn + 63) / 64 + 1) / 2), 1, (unsigned)batch);
    constexpr int kStateTile = 64 / kBwdStateLanes<N>;    // channels per wave of the state pass
    const dim3 state_grid((unsigned)(((a.Dn + kStateTile - 1) / kStateTile + 1) / 2), 1, (unsigned)batch);
    hipLaunchKernelGGL((bwd_state_kernel<N, IO, DENSE>), state_grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((bwd_kernel<N, IO, DENSE>), grid, dim3(256), 0, st, a);
}

template <int N, typename IO>
static void launch_form(bool dense, const BwdArgs& a, int batch, hipStream_t st)
{
    if (dense) launch_pair<N, IO, true>(a, batch, st);
    else launch_pair<N, IO, false>(a, batch, st);
}

void launch_bwd(int d_state, int io_bf16, bool dense, const BwdArgs& a, int batch, hipStream_t st)
{
#define BM_BWD(n)                                                \
    case n:                                                      \
        if (io_bf16) launch_form<n, IoBF16>(dense, a, batch, st); \
        else launch_form<n, IoF32>(dense, a, batch, st);          \
        break;
    switch (d_state) {
        BM_BWD(4)
        BM_BWD(8)
        BM_BWD(16)
        default: break;
    }
#undef BM_BWD
}

void launch_bwd_zero(float* p, long long n, hipStream_t st)
{
    if (!p || n <= 0) return;
    hipLaunchKernelGGL(bwd_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
}

}  // namespace bm
