// Instantiations of the scan kernels for one d_state (BM_N), compiled once per supported state size so the
// translation units build in parallel.
#include "kernels.h"
#include "launch.h"

#ifndef BM_N
#error "compile with -DBM_N=<d_state>"
#endif

namespace bm {

template <int AKIND, typename IO>
static void launch_one(const SweepArgs& sa, const CarryArgs& ca, dim3 grid, hipStream_t st, hipEvent_t ev_start,
                       hipEvent_t ev_stop)
{
    if (sa.nseg > 1) {
        hipLaunchKernelGGL((sweep_kernel<BM_N, AKIND, IO, kSummary>), grid, dim3(128), 0, st, sa);
        const long long threads = 2LL * ca.batch * ca.Dn;
        hipLaunchKernelGGL((carry_kernel<BM_N, AKIND>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ca);
    }
    if (ev_start) (void)hipEventRecord(ev_start, st);
    hipLaunchKernelGGL((sweep_kernel<BM_N, AKIND, IO, kSweep>), grid, dim3(128), 0, st, sa);
    if (ev_stop) (void)hipEventRecord(ev_stop, st);
}

#define BM_CAT2(a, b) a##b
#define BM_CAT(a, b) BM_CAT2(a, b)

void BM_CAT(launch_scan_n, BM_N)(int a_scalar_per_head, int io_bf16, const SweepArgs& sa, const CarryArgs& ca, dim3 grid,
                                 hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (a_scalar_per_head) {
        if (io_bf16) launch_one<1, IoBF16>(sa, ca, grid, st, ev_start, ev_stop);
        else launch_one<1, IoF32>(sa, ca, grid, st, ev_start, ev_stop);
    } else {
        if (io_bf16) launch_one<0, IoBF16>(sa, ca, grid, st, ev_start, ev_stop);
        else launch_one<0, IoF32>(sa, ca, grid, st, ev_start, ev_stop);
    }
}

}  // namespace bm
