// Instantiations and launchers of the chunked Mamba-2 kernels (d_state in {64, 128}, head width in {32, 64}).
#include "ssd_kernels.h"
#include "ssd_wide.h"
#include "launch.h"

#include <atomic>

namespace bm {

// Raising a kernel's dynamic-LDS limit is idempotent; it is done once per (kernel, device).
constexpr int kMaxDevices = 64;
static bool first_use_on_current_device(std::atomic<bool>* seen)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return true;
    return !seen[dev].exchange(true);
}

template <int N, int THREADS>
static void prep_variant(const SsdPrepPair& pa, int nchunk, int batch, hipStream_t st)
{
    static std::atomic<bool> seen[kMaxDevices];
    constexpr size_t lds = ssd_prep_lds_bytes<N, THREADS>();
    auto kernel = ssd_prep_kernel<N, THREADS>;
    if (first_use_on_current_device(seen))
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kernel, dim3((unsigned)nchunk, (unsigned)pa.dir[0].G, 2u * (unsigned)batch), dim3(THREADS), lds, st, pa);
}

template <int N, int P, bool SINGLE, int GROUPS, bool PARTS>
static void scan_variant(const SsdArgs& sa, int batch, hipStream_t st)
{
    static std::atomic<bool> seen[kMaxDevices];
    constexpr size_t lds = SsdLds<N, P, SINGLE>::bytes();
    auto kernel = ssd_kernel<N, P, SINGLE, GROUPS, PARTS>;
    if (first_use_on_current_device(seen))
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    const unsigned parts = !PARTS ? 1u : (unsigned)sa.parts;   // blockIdx.y is the time part
    hipLaunchKernelGGL(kernel, dim3((unsigned)sa.H, parts, (unsigned)batch), dim3(4 * P + 256 * GROUPS), lds, st, sa);
}

template <int N, int P>
static void wide_variant(const SsdArgs& sa, int batch, hipStream_t st)
{
    static std::atomic<bool> seen[kMaxDevices];
    constexpr size_t lds = SsdLds<N, P, false>::bytes();
    auto kernel = ssd_wide_kernel<N, P>;
    if (first_use_on_current_device(seen))
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kernel, dim3((unsigned)sa.H, 1, (unsigned)batch), dim3(SsdWide<N, P>::kThreads), lds, st, sa);
}

// Long calls that leave at least half of the CUs empty (batch 1 or 2) split the producers into two groups, which
// shortens the per-chunk chain of each workgroup (-4 to -9 %); with the chip full the extra waves only compete for
// issue slots (+4 to +7 %), so those keep one group.  (Calls of a single chunk go to launch_ssd_duo.)
template <int N, int P>
static void scan_one(const SsdArgs& sa, int batch, hipStream_t st)
{
    if (sa.wide) wide_variant<N, P>(sa, batch, st);
    else if (sa.parts > 1) scan_variant<N, P, false, 1, true>(sa, batch, st);
    else if (2LL * sa.H * batch <= cu_count()) scan_variant<N, P, false, 2, false>(sa, batch, st);
    else scan_variant<N, P, false, 1, false>(sa, batch, st);
}

bool ssd_supported(int d_state, int headdim) { return (d_state == 64 || d_state == 128) && (headdim == 32 || headdim == 64); }

// Launches that give a CU at most one workgroup take the sixteen-wave form: their duration is one workgroup's chain.
void launch_ssd_prep(int d_state, const SsdPrepPair& pa, int nchunk, int batch, hipStream_t st)
{
    const bool wide = 2LL * nchunk * pa.dir[0].G * batch <= cu_count();
    if (d_state == 128) {
        if (wide) prep_variant<128, 1024>(pa, nchunk, batch, st);
        else prep_variant<128, 256>(pa, nchunk, batch, st);
    } else {
        if (wide) prep_variant<64, 1024>(pa, nchunk, batch, st);
        else prep_variant<64, 256>(pa, nchunk, batch, st);
    }
}

void launch_ssd_carry(int d_state, const SsdCarryArgs& ca, hipStream_t st)
{
    const long long threads = 2LL * ca.batch * ca.Dn * d_state / 4;
    const dim3 grid((unsigned)((threads + 255) / 256));
    if (d_state == 128) hipLaunchKernelGGL(ssd_carry_kernel<128>, grid, dim3(256), 0, st, ca);
    else hipLaunchKernelGGL(ssd_carry_kernel<64>, grid, dim3(256), 0, st, ca);
}

template <int N, int P>
static void duo_one(const SsdStatePair& sp, int batch, hipStream_t st)
{
    static std::atomic<bool> seen[kMaxDevices];
    constexpr size_t lds = SsdDuoLds<N, P>::bytes();
    auto kernel = ssd_duo_kernel<N, P>;
    if (first_use_on_current_device(seen))
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kernel, dim3((unsigned)sp.dir[0].H, 1, (unsigned)batch), dim3(4 * P + 256), lds, st, sp);
}

// A call of one chunk: both directions of every (batch, head) item in one workgroup.
void launch_ssd_duo(int d_state, int headdim, const SsdStatePair& sp, int batch, hipStream_t st)
{
    if (d_state == 128 && headdim == 64) duo_one<128, 64>(sp, batch, st);
    else if (d_state == 128 && headdim == 32) duo_one<128, 32>(sp, batch, st);
    else if (d_state == 64 && headdim == 64) duo_one<64, 64>(sp, batch, st);
    else if (d_state == 64 && headdim == 32) duo_one<64, 32>(sp, batch, st);
}

// Both directions in one launch; nothing to do for the sub-part scanned last (no part starts after it).
void launch_ssd_state(int d_state, int headdim, const SsdStatePair& sp, int subs, int batch, hipStream_t st)
{
    if (subs < 2) return;
    const dim3 grid((unsigned)sp.dir[0].H, (unsigned)(subs - 1), (unsigned)(2 * batch));
    if (d_state == 128 && headdim == 64) hipLaunchKernelGGL((ssd_state_kernel<128, 64>), grid, dim3(256), 0, st, sp);
    else if (d_state == 128 && headdim == 32) hipLaunchKernelGGL((ssd_state_kernel<128, 32>), grid, dim3(256), 0, st, sp);
    else if (d_state == 64 && headdim == 64) hipLaunchKernelGGL((ssd_state_kernel<64, 64>), grid, dim3(256), 0, st, sp);
    else if (d_state == 64 && headdim == 32) hipLaunchKernelGGL((ssd_state_kernel<64, 32>), grid, dim3(256), 0, st, sp);
}

void launch_ssd_scan(int d_state, int headdim, const SsdArgs& sa, int batch, hipStream_t st)
{
    if (d_state == 128 && headdim == 64) scan_one<128, 64>(sa, batch, st);
    else if (d_state == 128 && headdim == 32) scan_one<128, 32>(sa, batch, st);
    else if (d_state == 64 && headdim == 64) scan_one<64, 64>(sa, batch, st);
    else if (d_state == 64 && headdim == 32) scan_one<64, 32>(sa, batch, st);
}

}  // namespace bm
