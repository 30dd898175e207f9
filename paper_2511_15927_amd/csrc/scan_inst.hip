// Instantiations of the scan kernels for one d_state (BM_N) and one lanes-per-chain factor (BM_S), compiled once per
// supported pair so the translation units build in parallel.
#include "kernels.h"
#include "launch.h"

#include <atomic>

#if !defined(BM_N) || !defined(BM_S)
#error "compile with -DBM_N=<d_state> -DBM_S=<lanes per chain>"
#endif

namespace bm {
namespace {  // this file is compiled once per (BM_N, BM_S): nothing below may be shared between those objects

// Even spread of a launch over the CUs.  The dispatcher places a workgroup wherever one fits, so a launch with fewer
// workgroups than the chip can hold ends up with some CUs full and others half empty, and the full ones set the
// kernel's duration.  Asking for a slice of LDS that nothing touches caps the workgroups resident on a CU at the
// number an even spread needs (per round, when the launch takes several), which makes the spread even.
constexpr int kLdsPerCu = 160 * 1024;
constexpr int kBlock = 256;
constexpr int kMaxDevices = 64;

static int current_device()
{
    int dev = 0;
    return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices ? dev : -1;
}

// What a CU holds of one kernel: workgroups resident at once (registers, static LDS) and the static LDS of each.
// Asked once per device; the same call lifts the kernel's dynamic-LDS limit to the whole CU, which the slices of
// launches with one or two workgroups per CU need.
struct KernelFit {
    std::atomic<int> resident[kMaxDevices];  // 0 = not asked yet
    std::atomic<int> static_lds[kMaxDevices];
    std::atomic<int> lifted[kMaxDevices];    // the raised limit took effect

    template <typename Kernel>
    int ask(Kernel kernel, int dev)
    {
        if (dev < 0) return 1;
        int r = resident[dev].load(std::memory_order_acquire);
        if (r == 0) {
            hipFuncAttributes fa;
            const void* fn = reinterpret_cast<const void*>(kernel);
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&r, kernel, kBlock, 0) != hipSuccess || r < 1) r = 1;
            const int fixed = hipFuncGetAttributes(&fa, fn) == hipSuccess ? (int)fa.sharedSizeBytes : 0;
            static_lds[dev].store(fixed, std::memory_order_relaxed);
            lifted[dev].store(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCu - fixed) == hipSuccess,
                              std::memory_order_relaxed);
            (void)hipGetLastError();
            resident[dev].store(r, std::memory_order_release);
        }
        return r;
    }
};

static long long workgroups_per_cu(const dim3& grid)
{
    const long long cus = cu_count();
    return ((long long)grid.x * grid.y * grid.z + cus - 1) / cus;
}

// How the waves that share a SIMD take turns at the issue priority (see take_turn): workgroups reach a CU in layers
// of one per CU, and a workgroup puts one wave on each SIMD, so a SIMD holds one wave per resident layer.
static SweepArgs with_turns(const SweepArgs& sa, const dim3& grid, int resident)
{
    SweepArgs s = sa;
    // Only when the whole launch is resident at once: with several rounds the workgroups start at different times
    // anyway and turns were measured to cost 5-6 %.
    const long long per_cu = workgroups_per_cu(grid);
    s.layer_wgs = cu_count();
    s.turn_mask = per_cu < 2 || per_cu > resident ? 0 : per_cu == 2 ? 1 : 3;
    return s;
}

static long long rounds(long long per_cu, int resident) { return (per_cu + resident - 1) / resident; }

// Bytes of dynamic LDS to ask for so that the launch spreads evenly (0: nothing to gain).
template <typename Kernel>
static unsigned spread_lds(Kernel kernel, KernelFit* fit, const dim3& grid)
{
    const int dev = current_device(), resident = fit->ask(kernel, dev);
    if (dev < 0) return 0;
    const long long per_cu = workgroups_per_cu(grid), n = rounds(per_cu, resident);
    const int cap = (int)((per_cu + n - 1) / n);
    if (cap >= resident) return 0;
    // between the largest slice of which cap + 1 fit and the largest of which cap fit
    const int slice = (kLdsPerCu / cap + kLdsPerCu / (cap + 1)) / 2 / 256 * 256;
    const int extra = slice - fit->static_lds[dev].load(std::memory_order_relaxed);
    if (extra < 0 || (slice > 64 * 1024 && !fit->lifted[dev].load(std::memory_order_relaxed))) return 0;
    return (unsigned)extra;
}

static dim3 sweep_grid(const SweepArgs& sa, int batch)
{
    constexpr int kCpw = 64 / BM_S;
    return dim3((unsigned)(((sa.Dn + kCpw - 1) / kCpw + 1) / 2), (unsigned)sa.nseg, (unsigned)batch);
}

template <int AKIND, typename IO, int TILE>
struct Tiled {
    static inline KernelFit fit_summary, fit_sweep;
    static constexpr auto summary = sweep_kernel<BM_N, BM_S, AKIND, IO, kSummary, TILE>;
    static constexpr auto sweep = sweep_kernel<BM_N, BM_S, AKIND, IO, kSweep, TILE>;

    static void launch(const SweepArgs& sa, const CarryArgs& ca, int batch, hipStream_t st, hipEvent_t ev_start,
                       hipEvent_t ev_stop)
    {
        const dim3 grid = sweep_grid(sa, batch);
        if (sa.nseg > 1) {
            hipLaunchKernelGGL(summary, grid, dim3(kBlock), spread_lds(summary, &fit_summary, grid), st,
                               with_turns(sa, grid, fit_summary.ask(summary, current_device())));
            const long long threads = 2LL * ca.batch * ca.Dn * BM_N;
            hipLaunchKernelGGL((carry_kernel<BM_N, AKIND>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ca);
        }
        const unsigned lds = spread_lds(sweep, &fit_sweep, grid);
        if (ev_start) (void)hipEventRecord(ev_start, st);
        hipLaunchKernelGGL(sweep, grid, dim3(kBlock), lds, st, with_turns(sa, grid, fit_sweep.ask(sweep, current_device())));
        if (ev_stop) (void)hipEventRecord(ev_stop, st);
    }
};

// One lane per chain and up to 32 states come with two prefetch depths: the deep tile hides memory latency when a
// SIMD holds few waves, the shallow one needs fewer registers, so more waves are resident at once.  The shallow tile
// is taken when it gets the launch through in fewer rounds of resident workgroups.
template <int AKIND, typename IO>
static void launch_one(const SweepArgs& sa, const CarryArgs& ca, int batch, int short_call, hipStream_t st,
                       hipEvent_t ev_start, hipEvent_t ev_stop)
{
#if BM_S == 1 && BM_N <= 16
    if (short_call) {   // one launch: the kernel converts the caller's B and C rows itself (see kBcStaged)
        const dim3 grid((unsigned)(((sa.Dn + 63) / 64 + 1) / 2), 1, (unsigned)batch);
        static KernelFit fit_short;
        auto sweep = sweep_kernel<BM_N, BM_S, AKIND, IO, kSweep, 8, kBcStaged>;
        const unsigned lds = spread_lds(sweep, &fit_short, grid);
        if (ev_start) (void)hipEventRecord(ev_start, st);
        hipLaunchKernelGGL(sweep, grid, dim3(kBlock), lds, st, with_turns(sa, grid, fit_short.ask(sweep, current_device())));
        if (ev_stop) (void)hipEventRecord(ev_stop, st);
        return;
    }
#endif
    (void)short_call;
    using Deep = Tiled<AKIND, IO, 8>;
#if BM_S == 1 && BM_N <= 32
    using Shallow = Tiled<AKIND, IO, 4>;
    const long long per_cu = workgroups_per_cu(sweep_grid(sa, batch));
    const int dev = current_device();
    if (rounds(per_cu, Shallow::fit_sweep.ask(Shallow::sweep, dev)) < rounds(per_cu, Deep::fit_sweep.ask(Deep::sweep, dev))) {
        Shallow::launch(sa, ca, batch, st, ev_start, ev_stop);
        return;
    }
#endif
    Deep::launch(sa, ca, batch, st, ev_start, ev_stop);
}

}  // namespace

#define BM_CAT4(a, b, c, d) a##b##c##d
#define BM_NAME(n, s) BM_CAT4(launch_scan_n, n, _s, s)

void BM_NAME(BM_N, BM_S)(int a_scalar_per_head, int io_bf16, const SweepArgs& sa, const CarryArgs& ca, int batch,
                         int short_call, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (a_scalar_per_head) {
        if (io_bf16) launch_one<1, IoBF16>(sa, ca, batch, short_call, st, ev_start, ev_stop);
        else launch_one<1, IoF32>(sa, ca, batch, short_call, st, ev_start, ev_stop);
    } else {
        if (io_bf16) launch_one<0, IoBF16>(sa, ca, batch, short_call, st, ev_start, ev_stop);
        else launch_one<0, IoF32>(sa, ca, batch, short_call, st, ev_start, ev_stop);
    }
}

}  // namespace bm
