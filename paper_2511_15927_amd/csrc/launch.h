// Host-callable launchers of the scan kernels (defined in scan_inst.hip, one object per (d_state, lanes-per-chain)).
#pragma once
#include "kernels.h"

namespace bm {
// Compute units of the current device (256 when no device answers), asked once per device; defined in bimamba_api.hip
// and used by the host-side plan and by every launcher, so that all of them size a launch for the same chip.
int cu_count();

#define BM_DECLARE_SCAN(n, s)                                                                                      \
    void launch_scan_n##n##_s##s(int a_scalar_per_head, int io_bf16, const SweepArgs& sa, const CarryArgs& ca,     \
                                 int batch, int short_call, hipStream_t st, hipEvent_t ev_start,                   \
                                 hipEvent_t ev_stop);
BM_DECLARE_SCAN(4, 1)
BM_DECLARE_SCAN(8, 1)
BM_DECLARE_SCAN(16, 1)
BM_DECLARE_SCAN(16, 2)
BM_DECLARE_SCAN(16, 4)
BM_DECLARE_SCAN(32, 1)
BM_DECLARE_SCAN(32, 2)
BM_DECLARE_SCAN(32, 4)
BM_DECLARE_SCAN(64, 1)
BM_DECLARE_SCAN(64, 4)
BM_DECLARE_SCAN(128, 1)
BM_DECLARE_SCAN(128, 4)
#undef BM_DECLARE_SCAN

struct SsdPrepPair;
struct SsdArgs;
struct SsdCarryArgs;
struct SsdStatePair;
bool ssd_supported(int d_state, int headdim);
void launch_ssd_prep(int d_state, const SsdPrepPair& pa, int nchunk, int batch, hipStream_t st);
void launch_ssd_scan(int d_state, int headdim, const SsdArgs& sa, int batch, hipStream_t st);
void launch_ssd_carry(int d_state, const SsdCarryArgs& ca, hipStream_t st);
void launch_ssd_duo(int d_state, int headdim, const SsdStatePair& sp, int batch, hipStream_t st);
void launch_ssd_state(int d_state, int headdim, const SsdStatePair& sp, int subs, int batch, hipStream_t st);

struct BwdArgs;
struct BwdBcArgs;
void launch_bwd_bc(const BwdBcArgs& a, hipStream_t st);
bool bwd_supported(int d_state);
int bwd_chunk_tokens(int d_state, bool dense);
bool bwd_dense(int d_inner, int batch);
void launch_bwd(int d_state, int io_bf16, bool dense, const BwdArgs& a, int batch, hipStream_t st);
void launch_bwd_zero(float* p, long long n, hipStream_t st);
}  // namespace bm
