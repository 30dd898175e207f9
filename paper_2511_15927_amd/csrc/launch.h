// Host-callable launchers of the per-d_state scan kernels (defined in scan_inst.hip, one object per d_state).
#pragma once
#include "kernels.h"

namespace bm {
#define BM_DECLARE_SCAN(n) \
    void launch_scan_n##n(int a_scalar_per_head, int io_bf16, const SweepArgs& sa, const CarryArgs& ca, dim3 grid, hipStream_t st, \
                          hipEvent_t ev_start, hipEvent_t ev_stop);
BM_DECLARE_SCAN(4)
BM_DECLARE_SCAN(8)
BM_DECLARE_SCAN(16)
BM_DECLARE_SCAN(32)
BM_DECLARE_SCAN(64)
BM_DECLARE_SCAN(128)
#undef BM_DECLARE_SCAN
}  // namespace bm
