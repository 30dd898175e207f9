// Instantiations of the scan kernels for one d_state (BM_N) and one lanes-per-chain factor (BM_S), compiled once per
// supported pair so the translation units build in parallel.
#include "kernels.h"
#include "launch.h"

#if !defined(BM_N) || !defined(BM_S)
#error "compile with -DBM_N=<d_state> -DBM_S=<lanes per chain>"
#endif

namespace bm {

template <int AKIND, typename IO, int TILE>
static void launch_tile(const SweepArgs& sa, const CarryArgs& ca, int batch, hipStream_t st, hipEvent_t ev_start,
                        hipEvent_t ev_stop)
{
    constexpr int kCpw = 64 / BM_S;
    const dim3 grid((unsigned)((sa.Dn + kCpw - 1) / kCpw), (unsigned)sa.nseg, (unsigned)batch);
    if (sa.nseg > 1) {
        hipLaunchKernelGGL((sweep_kernel<BM_N, BM_S, AKIND, IO, kSummary, TILE>), grid, dim3(128), 0, st, sa);
        const long long threads = 2LL * ca.batch * ca.Dn;
        hipLaunchKernelGGL((carry_kernel<BM_N, AKIND>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ca);
    }
    if (ev_start) (void)hipEventRecord(ev_start, st);
    hipLaunchKernelGGL((sweep_kernel<BM_N, BM_S, AKIND, IO, kSweep, TILE>), grid, dim3(128), 0, st, sa);
    if (ev_stop) (void)hipEventRecord(ev_stop, st);
}

// Shallow tiles exist for one lane per chain and up to 32 states (the case with enough chains for four or more waves
// per SIMD); every other instantiation uses the deep tile.
template <int AKIND, typename IO>
static void launch_one(const SweepArgs& sa, const CarryArgs& ca, int batch, int shallow_tile, int short_call,
                       hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop)
{
#if BM_S == 1 && BM_N <= 16
    if (short_call) {   // one launch: the kernel converts the caller's B and C rows itself (see kBcStaged)
        const dim3 grid((unsigned)((sa.Dn + 63) / 64), 1, (unsigned)batch);
        if (ev_start) (void)hipEventRecord(ev_start, st);
        hipLaunchKernelGGL((sweep_kernel<BM_N, BM_S, AKIND, IO, kSweep, 8, kBcStaged>), grid, dim3(128), 0, st, sa);
        if (ev_stop) (void)hipEventRecord(ev_stop, st);
        return;
    }
#endif
    (void)short_call;
#if BM_S == 1 && BM_N <= 32
    if (shallow_tile) {
        launch_tile<AKIND, IO, 4>(sa, ca, batch, st, ev_start, ev_stop);
        return;
    }
#endif
    (void)shallow_tile;
    launch_tile<AKIND, IO, 8>(sa, ca, batch, st, ev_start, ev_stop);
}

#define BM_CAT4(a, b, c, d) a##b##c##d
#define BM_NAME(n, s) BM_CAT4(launch_scan_n, n, _s, s)

void BM_NAME(BM_N, BM_S)(int a_scalar_per_head, int io_bf16, const SweepArgs& sa, const CarryArgs& ca, int batch,
                         int shallow_tile, int short_call, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (a_scalar_per_head) {
        if (io_bf16) launch_one<1, IoBF16>(sa, ca, batch, shallow_tile, short_call, st, ev_start, ev_stop);
        else launch_one<1, IoF32>(sa, ca, batch, shallow_tile, short_call, st, ev_start, ev_stop);
    } else {
        if (io_bf16) launch_one<0, IoBF16>(sa, ca, batch, shallow_tile, short_call, st, ev_start, ev_stop);
        else launch_one<0, IoF32>(sa, ca, batch, shallow_tile, short_call, st, ev_start, ev_stop);
    }
}

}  // namespace bm
