// Host side of the C ABI declared in include/bimamba.h: argument validation, workspace carving, kernel dispatch.
#include "bimamba.h"
#include "kernels.h"
#include "launch.h"
#include "bwd_kernels.h"
#include "ssd_kernels.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>

// Device memory of bimamba_block_fwd_static, the entry point for callers that cannot allocate: one copy per GPU, held
// until the process ends.  In host code this name only identifies the symbol; the address a kernel can use is asked
// from the runtime once per device (static_scratch below).
static __device__ __align__(256) unsigned char scratch[BIMAMBA_STATIC_SCRATCH_BYTES];

namespace {

using namespace bm;

thread_local hipEvent_t g_probe_start = nullptr, g_probe_stop = nullptr;  // one-shot, see bimamba_profile_next_call

}  // namespace

namespace bm {
int cu_count()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) {
        cus = cached[dev].load(std::memory_order_relaxed);
        if (cus == 0) {
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
            cached[dev].store(cus, std::memory_order_relaxed);
        }
    }
    return cus;   // no device (a host-only query): plan for the 256-CU chip
}
}  // namespace bm

namespace {

// Launch geometry is planned for the SIMDs the device has (four per CU); the thresholds below were measured on MI355X
// (256 CUs, 1024 SIMDs).
inline int simds() { return 4 * cu_count(); }
inline int target_waves() { return 2 * simds(); }   // two waves per SIMD

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Byte range [lo, hi) a tensor view spans (non-negative strides, checked before this is used).
struct Span {
    uintptr_t lo, hi;
};
Span span_of(const bimamba_tensor& t, int channels, size_t elem, const bimamba_desc* d)
{
    const uintptr_t lo = reinterpret_cast<uintptr_t>(t.ptr);
    const int64_t last = (int64_t)(d->batch - 1) * t.stride_batch + (int64_t)(d->seqlen - 1) * t.stride_token + channels;
    return Span{lo, lo + (uintptr_t)last * elem};
}

// Whether writing `out` could touch memory an input view reads.  Views whose byte ranges are apart never do; views
// that interleave inside one buffer (column slices of one projection output, the usual layout) do not either when
// they share both strides, rows tile the batch stride, and their column ranges are apart modulo the row pitch.
bool may_overlap(const bimamba_tensor& out, int out_ch, const bimamba_tensor& in, int in_ch, size_t elem,
                 const bimamba_desc* d)
{
    const Span a = span_of(out, out_ch, elem, d), b = span_of(in, in_ch, elem, d);
    if (a.hi <= b.lo || b.hi <= a.lo) return false;
    if (out.stride_token == in.stride_token && out.stride_batch == in.stride_batch && out.stride_token > 0 &&
        out.stride_batch % out.stride_token == 0) {
        const int64_t pitch = out.stride_token;
        const int64_t delta = ((int64_t)a.lo - (int64_t)b.lo) / (int64_t)elem;
        const int64_t r = ((delta % pitch) + pitch) % pitch;   // out's first column, counted from in's first column
        if (r >= in_ch && r + out_ch <= pitch) return false;
    }
    return true;
}
inline bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

__global__ __launch_bounds__(256) void zero_fill_kernel(float* p, long long n)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

bool split_supported(int d_state, int split)
{
    switch (d_state * 8 + split) {
        case 4 * 8 + 1: case 8 * 8 + 1: case 16 * 8 + 1: case 16 * 8 + 2: case 16 * 8 + 4: case 32 * 8 + 1:
        case 32 * 8 + 2: case 32 * 8 + 4: case 64 * 8 + 1: case 64 * 8 + 4: case 128 * 8 + 1: case 128 * 8 + 4:
            return true;
        default: return false;
    }
}

int check_desc(const bimamba_desc* d)
{
    if (!d) return BIMAMBA_ERR_NULL_POINTER;
    if (d->struct_size != sizeof(bimamba_desc)) return BIMAMBA_ERR_BAD_SHAPE;
    if (d->batch < 0 || d->seqlen < 0 || d->d_inner < 1 || d->d_state < 1 || d->n_heads < 1 || d->n_groups < 1 ||
        d->d_conv < 1)
        return BIMAMBA_ERR_BAD_SHAPE;
    if (d->d_inner % d->n_heads || d->n_heads % d->n_groups) return BIMAMBA_ERR_BAD_SHAPE;
    if (d->time_chunks < 0 || d->state_split < 0) return BIMAMBA_ERR_BAD_SHAPE;
    if (d->state_split > 0 && !split_supported(d->d_state, d->state_split)) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->batch > 65535) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->io_dtype != BIMAMBA_F32 && d->io_dtype != BIMAMBA_BF16) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->a_kind != BIMAMBA_A_PER_HEAD_STATE && d->a_kind != BIMAMBA_A_SCALAR_PER_HEAD) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->d_kind != BIMAMBA_D_PER_CHANNEL && d->d_kind != BIMAMBA_D_PER_HEAD) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->combine != BIMAMBA_COMBINE_ADD && d->combine != BIMAMBA_COMBINE_SEPARATE) return BIMAMBA_ERR_UNSUPPORTED;
    if ((d->dt_softplus | 1) != 1 || (d->conv_bc | 1) != 1) return BIMAMBA_ERR_UNSUPPORTED;
    if (d->d_conv > 4) return BIMAMBA_ERR_UNSUPPORTED;
    switch (d->d_state) {
        case 4: case 8: case 16: case 32: case 64: case 128: break;
        default: return BIMAMBA_ERR_UNSUPPORTED;
    }
    if (d->n_groups > 1 && (d->d_inner / d->n_groups) % 64 != 0) return BIMAMBA_ERR_UNSUPPORTED;
    return BIMAMBA_OK;
}

long long waves_of(const bimamba_desc* d, int split)
{
    const int cpw = 64 / split;
    return 2LL * d->batch * ((d->d_inner + cpw - 1) / cpw);
}

// Launch geometry of the lane-per-chain kernels, from measurements on MI355X (1024 SIMDs) with w = the number of waves
// that one lane per chain gives (2 * batch * d_inner / 64), up to 32 states:
//   first       two lanes per chain (each holds half the states), whole sequence, when the 2w waves fill the rounds of
//               resident waves well (two_lanes_fit below).
//   w >= 1920   one lane per chain, whole sequence: close to two waves per SIMD already.
//   else        one lane per chain and the sequence cut into time segments until about 16 waves per SIMD exist: the
//               segment summaries cost a second, cheaper pass, but every SIMD then holds enough waves to issue back
//               to back and to hide the loads, whatever the batch.  Segments stay at 256 tokens or more when that
//               still gives four waves per SIMD, at 128 or more otherwise.
//               If even that leaves fewer than two waves per SIMD (short sequences), two lanes per chain.
// Four lanes per chain cost as many vector instructions per channel and token as two (measured with the tokens dealt:
// 2.36 ms against 1.83 at the headline shape, and twice the HBM fetch because four tiles share a 128-byte line) and
// are not picked below 64 states.  With 64 or 128 states a lane cannot hold a whole chain without starving the SIMD of
// registers, so those shapes split the states first (four lanes per chain) and cut the sequence only as far as two
// waves per SIMD need, in segments of at least 256 tokens.
constexpr int kWavesForSegments = 16384;
constexpr int kMinSegmentTokens = 128;

bool many_states(const bimamba_desc* d) { return d->d_state > 32; }

int segments_for(const bimamba_desc* d, long long waves)
{
    const int L = d->seqlen;
    if (L <= 0 || waves <= 0) return 1;
    const int want = many_states(d) ? target_waves() : kWavesForSegments;
    long long min_tokens = 256;
    if (!many_states(d) && waves * (L / 256) < 4 * simds()) min_tokens = kMinSegmentTokens;
    long long n = (want + waves - 1) / waves;
    const long long max_by_len = L / min_tokens > 0 ? L / min_tokens : 1;
    if (n > max_by_len) n = max_by_len;
    return (int)(n < 1 ? 1 : n);
}

// Two lanes per chain, whole sequence.  Up to 16 states the pair deals its tokens (see run_tiles_dealt) and a SIMD
// holds three such waves at once: measured at d_inner 4096 (L 8192, batch 5 to 32) and d_inner 2048 (L 1024 to 8192,
// batch 16 to 64) against the best of the other geometries, it wins from 1.7 to 5 waves per SIMD (batch 7 to 20 at
// d_inner 4096: -3 to -23 %) and loses outside.
// With 32 states the plain walk keeps three waves on a SIMD: 1.8 to 2, or 2.35 to 3 per SIMD.
bool two_lanes_fit(const bimamba_desc* d, long long w)
{
    const long long per_simd_x100 = 2 * w * 100 / simds();
    if (d->d_state <= 16) return per_simd_x100 >= 170 && per_simd_x100 <= 500;
    return (per_simd_x100 >= 180 && per_simd_x100 <= 200) || (per_simd_x100 >= 235 && per_simd_x100 <= 300);
}

// One lane per chain needs no help from segments or lane splitting.
bool enough_chains(const bimamba_desc* d, long long w) { return many_states(d) ? w >= target_waves() : 8 * w >= 15 * simds(); }

int pick_split(const bimamba_desc* d)
{
    if (d->state_split > 0) return d->state_split;
    const long long w = waves_of(d, 1);
    const bool two = split_supported(d->d_state, 2), four = d->d_state >= 64 && split_supported(d->d_state, 4);
    // (calls of a few dozen tokens that can run as one launch with one lane per chain keep it, see short_call below:
    // 32-token block steps at batch 16, d_inner 4096 take 23 us that way against 28 us with two lanes and a preparation launch)
    const bool one_launch_form = d->d_state <= 16 && !d->conv_bc && d->seqlen <= kShortCallTokens && enough_chains(d, w);
    if (!many_states(d) && two && d->time_chunks <= 1 && !one_launch_form && two_lanes_fit(d, w)) return 2;
    if (enough_chains(d, w)) return 1;
    if (many_states(d)) return w >= target_waves() / 2 && two ? 2 : four ? 4 : two ? 2 : 1;
    if (d->time_chunks == 0 && w * segments_for(d, w) >= target_waves()) return 1;
    return two ? 2 : 1;
}

int pick_chunks(const bimamba_desc* d, int split)
{
    const int L = d->seqlen;
    if (L <= 0) return 1;
    int n;
    if (d->time_chunks > 0) {
        n = d->time_chunks;
    } else {
        const long long waves = waves_of(d, split);
        const long long w = waves_of(d, 1);
        const bool whole = d->state_split == 0 && !many_states(d) &&
                           (split == 1 ? enough_chains(d, w) : split == 2 && two_lanes_fit(d, w));
        n = waves >= target_waves() || whole ? 1 : segments_for(d, waves);
    }
    if (n > L) n = L;
    if (n > 4096) n = 4096;
    if (n < 1) n = 1;
    return n;
}

struct Plan {
    int split, nseg, seg_len;
    bool two_bc;  // the two directions consume different prepared B|C buffers
    bool ssd;     // Mamba-2 parameterisation on the chunked matrix-core kernels
    int ssd_chunks;
    int ssd_parts, ssd_part_chunks;  // time parts of the matrix-core path (1: every (batch, head) item is one workgroup)
    int ssd_subs, ssd_part_subs, ssd_sub_chunks;  // sub-parts the state pass walks: in all, per part, chunks of each
    size_t off_bc[2], off_partial, off_carry, off_sumdt, off_crows[2], off_bt[2], off_score[2], off_pstate[2], off_pdecay[2], total;
};

// The chunked matrix-core path covers bf16 I/O with one decay rate per head, d_state 64 or 128 and heads of 32 or
// 64 channels; forcing time_chunks or state_split selects the lane-per-chain kernels instead.
bool use_ssd(const bimamba_desc* d)
{
    return d->a_kind == BIMAMBA_A_SCALAR_PER_HEAD && d->io_dtype == BIMAMBA_BF16 && d->time_chunks == 0 &&
           d->state_split == 0 && ssd_supported(d->d_state, d->d_inner / d->n_heads) &&
           d->batch <= 32767;   // the preparation kernel's grid holds both directions of every batch element
}

Plan make_plan(const bimamba_desc* d, bool inputs_shared)
{
    Plan p{};
    // The lane-per-chain geometry is always planned (and its workspace reserved): a call whose x tensors do not meet
    // the matrix-core kernels' alignment needs falls back to it.
    p.ssd = use_ssd(d);
    p.split = pick_split(d);
    p.nseg = pick_chunks(d, p.split);
    p.seg_len = d->seqlen > 0 ? (d->seqlen + p.nseg - 1) / p.nseg : 1;
    p.nseg = d->seqlen > 0 ? (d->seqlen + p.seg_len - 1) / p.seg_len : 1;
    p.two_bc = d->conv_bc || !inputs_shared;
    const size_t bc_bytes = align_up((size_t)d->batch * d->seqlen * d->n_groups * 2 * d->d_state * sizeof(float), 256);
    size_t off = 0;
    p.off_bc[0] = off; off += bc_bytes;
    if (p.two_bc) { p.off_bc[1] = off; off += bc_bytes; } else { p.off_bc[1] = p.off_bc[0]; }
    p.off_partial = off;
    if (d->combine == BIMAMBA_COMBINE_ADD) off += align_up((size_t)d->batch * d->seqlen * d->d_inner * sizeof(float), 256);
    p.off_carry = off;
    p.off_sumdt = off;
    if (p.nseg > 1) {
        off += align_up((size_t)2 * d->batch * p.nseg * d->d_inner * d->d_state * sizeof(float), 256);
        p.off_sumdt = off;
        off += align_up((size_t)2 * d->batch * p.nseg * d->d_inner * sizeof(float), 256);
    }
    p.ssd_chunks = (d->seqlen + kQ - 1) / kQ;
    // Time parts: a call whose (batch, head) items would leave at least half of the 256 CUs empty deals each item's
    // chunks to several workgroups (at least 8 chunks each, at most 16 parts); a first, cheaper pass then finds the
    // state entering each part.  That pass runs light workgroups, four to a CU, so it cuts the parts further into
    // sub-parts (at least 4 chunks each) until both directions together bring about that many.
    p.ssd_parts = p.ssd_subs = p.ssd_part_subs = 1;
    p.ssd_part_chunks = p.ssd_sub_chunks = p.ssd_chunks;
    if (p.ssd) {
        const long long items = (long long)d->n_heads * d->batch;
        const int cus = cu_count();
        long long parts = items > 0 ? cus / items : 1;
        if (parts > p.ssd_chunks / 8) parts = p.ssd_chunks / 8;
        if (parts > 16) parts = 16;
        if (parts >= 2) {
            const int part_chunks = (int)((p.ssd_chunks + parts - 1) / parts);
            const long long subs_wanted = (4LL * cus + 2 * items - 1) / (2 * items);
            long long k = (subs_wanted + parts - 1) / parts;
            if (k > part_chunks / 4) k = part_chunks / 4;
            if (k < 1) k = 1;
            p.ssd_part_subs = (int)k;
            p.ssd_sub_chunks = (int)((part_chunks + k - 1) / k);
            p.ssd_part_chunks = p.ssd_part_subs * p.ssd_sub_chunks;
            p.ssd_parts = (p.ssd_chunks + p.ssd_part_chunks - 1) / p.ssd_part_chunks;
            p.ssd_subs = (p.ssd_chunks + p.ssd_sub_chunks - 1) / p.ssd_sub_chunks;
        }
    }
    if (p.ssd) {
        const size_t rows = align_up((size_t)d->batch * p.ssd_chunks * kQ * d->n_groups * d->d_state * sizeof(__bf16), 256);
        const size_t score = align_up((size_t)d->batch * p.ssd_chunks * d->n_groups * kScoreOp * sizeof(float), 256);
        for (int s = 0; s < 2; s++) {
            p.off_crows[s] = off; off += rows;
            p.off_bt[s] = off; off += rows;
            p.off_score[s] = off; off += score;
        }
        for (int s = 0; s < 2; s++) {
            p.off_pstate[s] = p.off_pdecay[s] = off;
            if (p.ssd_parts > 1) {
                off += align_up((size_t)p.ssd_subs * d->batch * d->d_inner * d->d_state * sizeof(float), 256);
                p.off_pdecay[s] = off;
                off += align_up((size_t)p.ssd_subs * d->batch * d->n_heads * sizeof(float), 256);
            }
        }
    }
    p.total = off;
    return p;
}

constexpr int64_t kMaxTokenStride = 1 << 26;  // elements

int check_tensor(const bimamba_tensor& t, int channels, size_t elem, const bimamba_desc* d)
{
    const bool empty = d->batch == 0 || d->seqlen == 0;  // nothing is read or written: the pointer may be NULL
    if (!t.ptr && !empty) return BIMAMBA_ERR_NULL_POINTER;
    if (!is_aligned(t.ptr, elem)) return BIMAMBA_ERR_MISALIGNED;
    if (empty) return BIMAMBA_OK;                         // no element exists, so no stride is ever used
    if (t.stride_token < channels) return BIMAMBA_ERR_BAD_SHAPE;
    if (t.stride_token > kMaxTokenStride) return BIMAMBA_ERR_UNSUPPORTED;  // row offsets inside a tile are 32-bit
    if (d->batch > 1 && t.stride_batch < (int64_t)d->seqlen * t.stride_token - (t.stride_token - channels))
        return BIMAMBA_ERR_BAD_SHAPE;
    return BIMAMBA_OK;
}

int check_params(const bimamba_params* p)
{
    if (!p) return BIMAMBA_ERR_NULL_POINTER;
    if (!p->conv_w || !p->A || !p->D) return BIMAMBA_ERR_NULL_POINTER;
    if (!is_aligned(p->conv_w, 4) || !is_aligned(p->A, 4) || !is_aligned(p->D, 4) || !is_aligned(p->conv_b, 4) ||
        !is_aligned(p->dt_bias, 4))
        return BIMAMBA_ERR_MISALIGNED;
    return BIMAMBA_OK;
}

int check_inputs(const bimamba_inputs* in, const bimamba_desc* d, size_t elem)
{
    if (!in) return BIMAMBA_ERR_NULL_POINTER;
    int rc;
    if ((rc = check_tensor(in->x, d->d_inner, elem, d))) return rc;
    if ((rc = check_tensor(in->z, d->d_inner, elem, d))) return rc;
    if ((rc = check_tensor(in->dt, d->n_heads, elem, d))) return rc;
    if ((rc = check_tensor(in->B, d->n_groups * d->d_state, elem, d))) return rc;
    if ((rc = check_tensor(in->C, d->n_groups * d->d_state, elem, d))) return rc;
    return BIMAMBA_OK;
}

bool same_tensor(const bimamba_tensor& a, const bimamba_tensor& b)
{
    return a.ptr == b.ptr && a.stride_batch == b.stride_batch && a.stride_token == b.stride_token;
}

bool same_inputs(const bimamba_inputs* a, const bimamba_inputs* b)
{
    return a == b || (same_tensor(a->x, b->x) && same_tensor(a->z, b->z) && same_tensor(a->dt, b->dt) &&
                      same_tensor(a->B, b->B) && same_tensor(a->C, b->C));
}

bool pairs_readable(const bimamba_tensor& t)
{
    return is_aligned(t.ptr, 4) && t.stride_batch % 2 == 0 && t.stride_token % 2 == 0;
}

TensorArg targ(const bimamba_tensor& t) { return TensorArg{t.ptr, (long long)t.stride_batch, (long long)t.stride_token}; }

// A call of a few dozen tokens with one lane per chain, up to 16 states and no conv on B and C runs as a single
// launch: the scan kernel converts the caller's B and C rows itself instead of reading prepared fp32 rows.
bool short_call(const bimamba_desc* d, const Plan& plan)
{
    return !plan.ssd && plan.split == 1 && plan.nseg == 1 && d->d_state <= 16 && !d->conv_bc &&
           d->seqlen <= kShortCallTokens;
}

void launch_scan(const bimamba_desc* d, int split, int short_call, const SweepArgs& sa, const CarryArgs& ca,
                 hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    const int scalar_a = d->a_kind == BIMAMBA_A_SCALAR_PER_HEAD, bf16 = d->io_dtype == BIMAMBA_BF16;
#define BM_CASE(n, s) \
    case (n) * 8 + (s):                                                                                          \
        launch_scan_n##n##_s##s(scalar_a, bf16, sa, ca, d->batch, short_call, st, ev_start, ev_stop);              \
        break;
    switch (d->d_state * 8 + split) {
        BM_CASE(4, 1) BM_CASE(8, 1) BM_CASE(16, 1) BM_CASE(16, 2) BM_CASE(16, 4) BM_CASE(32, 1) BM_CASE(32, 2)
        BM_CASE(32, 4) BM_CASE(64, 1) BM_CASE(64, 4) BM_CASE(128, 1) BM_CASE(128, 4)
        default: break;
    }
#undef BM_CASE
}

int run(const bimamba_desc* d, const bimamba_params* pf, const bimamba_params* pb, const bimamba_inputs* in_f,
        const bimamba_inputs* in_b, const float* h_in, const void* tail_in, float* h_out, void* tail_out,
        const bimamba_tensor* out, void* workspace, size_t workspace_bytes, void* hip_stream, bool block_variant)
{
    const hipEvent_t probe_start = g_probe_start, probe_stop = g_probe_stop;
    g_probe_start = g_probe_stop = nullptr;
    int rc = check_desc(d);
    if (rc) return rc;
    const size_t elem = d->io_dtype == BIMAMBA_BF16 ? 2 : 4;
    if ((rc = check_params(pf))) return rc;
    if ((rc = check_params(pb))) return rc;
    if (!in_b) in_b = in_f;
    if ((rc = check_inputs(in_f, d, elem))) return rc;
    if ((rc = check_inputs(in_b, d, elem))) return rc;
    if (!out) return BIMAMBA_ERR_NULL_POINTER;
    const int out_ch = d->combine == BIMAMBA_COMBINE_SEPARATE ? 2 * d->d_inner : d->d_inner;
    if ((rc = check_tensor(*out, out_ch, elem, d))) return rc;
    if (!is_aligned(h_in, 4) || !is_aligned(h_out, 4) || !is_aligned(tail_in, elem) || !is_aligned(tail_out, elem))
        return BIMAMBA_ERR_MISALIGNED;
    const bool shared = same_inputs(in_f, in_b);
    Plan plan = make_plan(d, shared);
    // the chunked kernels read x two channels at a time and the carried state four states at a time
    if (plan.ssd && !(pairs_readable(in_f->x) && pairs_readable(in_b->x) && is_aligned(h_in, 16) && is_aligned(h_out, 16)))
        plan.ssd = false;
    // the state pass of the time parts addresses the 67 token rows of a chunk with 32-bit byte offsets
    constexpr int64_t kMaxPartsTokenStride = 1 << 24;
    if (plan.ssd && plan.ssd_parts > 1 &&
        (in_f->x.stride_token > kMaxPartsTokenStride || in_b->x.stride_token > kMaxPartsTokenStride)) {
        plan.ssd_parts = plan.ssd_subs = plan.ssd_part_subs = 1;
        plan.ssd_part_chunks = plan.ssd_sub_chunks = plan.ssd_chunks;
    }
    if (plan.total > 0) {
        if (!workspace) return BIMAMBA_ERR_NULL_POINTER;
        if (!is_aligned(workspace, 16)) return BIMAMBA_ERR_MISALIGNED;
        if (workspace_bytes < plan.total) return BIMAMBA_ERR_WORKSPACE_TOO_SMALL;
    }
    if (d->batch > 0 && d->seqlen > 0) {
        const int gn = d->n_groups * d->d_state;
        for (const bimamba_inputs* in : {in_f, in_b}) {
            if (may_overlap(*out, out_ch, in->x, d->d_inner, elem, d) || may_overlap(*out, out_ch, in->z, d->d_inner, elem, d) ||
                may_overlap(*out, out_ch, in->dt, d->n_heads, elem, d) || may_overlap(*out, out_ch, in->B, gn, elem, d) ||
                may_overlap(*out, out_ch, in->C, gn, elem, d))
                return BIMAMBA_ERR_ALIAS;
        }
    }
    const hipError_t pending = hipPeekAtLastError();   // an error some earlier, unrelated call left behind is not ours to report or clear
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int GN = d->n_groups * d->d_state;
    const int tail_ch = d->d_inner + (d->conv_bc ? 2 * GN : 0);
    char* ws = static_cast<char*>(workspace);

    if (d->batch > 0 && d->seqlen > 0) {
        // 1. fp32 B|C rows per direction (the chunked path prepares its own operand tiles from the raw rows)
        const bool one_launch = short_call(d, plan);
        const int nbuf = (plan.ssd || one_launch) ? 0 : plan.two_bc ? 2 : 1;
        for (int s = 0; s < nbuf; s++) {
            const bimamba_inputs* in = s == 0 ? in_f : in_b;
            const bimamba_params* p = s == 0 ? pf : pb;
            PrepArgs pa{};
            pa.B = targ(in->B);
            pa.C = targ(in->C);
            pa.conv_w = p->conv_w;
            pa.conv_b = p->conv_b;
            pa.tail_in = (s == 0 && block_variant) ? tail_in : nullptr;
            pa.dst = reinterpret_cast<float*>(ws + plan.off_bc[s]);
            pa.batch = d->batch; pa.L = d->seqlen; pa.G = d->n_groups; pa.N = d->d_state; pa.K = d->d_conv;
            pa.Dn = d->d_inner; pa.tail_ch = tail_ch; pa.conv_bc = d->conv_bc; pa.dir = s == 0 ? 1 : -1;
            const long long total = (long long)d->batch * d->seqlen * 2 * GN;
            const dim3 grid((unsigned)((total + 255) / 256));
            if (d->io_dtype == BIMAMBA_BF16) hipLaunchKernelGGL(prep_bc_kernel<IoBF16>, grid, dim3(256), 0, st, pa);
            else hipLaunchKernelGGL(prep_bc_kernel<IoF32>, grid, dim3(256), 0, st, pa);
        }
        if (plan.ssd) {
            // 2'. chunked matrix-core path: per-direction operand tiles, then the reverse scan parks its result and the
            // forward scan adds, gates and stores (or each writes its own half)
            const bool separate = d->combine == BIMAMBA_COMBINE_SEPARATE;
            const bool raw = !separate && same_tensor(in_f->z, in_b->z);
            SsdPrepPair pp{};
            for (int s = 0; s < 2; s++) {
                SsdPrepArgs& pa = pp.dir[s];
                const bimamba_inputs* in = s == 0 ? in_f : in_b;
                const bimamba_params* p = s == 0 ? pf : pb;
                pa.B = targ(in->B); pa.C = targ(in->C);
                pa.conv_w = p->conv_w; pa.conv_b = p->conv_b;
                pa.tail_in = (s == 0 && block_variant) ? tail_in : nullptr;
                pa.K = d->d_conv; pa.Dn = d->d_inner; pa.tail_ch = tail_ch; pa.conv_bc = d->conv_bc;
                pa.c_rows = reinterpret_cast<__bf16*>(ws + plan.off_crows[s]);
                pa.b_t = reinterpret_cast<__bf16*>(ws + plan.off_bt[s]);
                pa.score_op = reinterpret_cast<float*>(ws + plan.off_score[s]);
                pa.L = d->seqlen; pa.G = d->n_groups; pa.dir = s == 0 ? 1 : -1;
            }
            launch_ssd_prep(d->d_state, pp, plan.ssd_chunks, d->batch, st);
            if (probe_start) (void)hipEventRecord(probe_start, st);
            auto scan_args = [&](int s) {
                const bimamba_inputs* in = s == 0 ? in_f : in_b;
                const bimamba_params* p = s == 0 ? pf : pb;
                SsdArgs sa{};
                sa.x = targ(in->x); sa.z = targ(in->z); sa.dt = targ(in->dt);
                sa.conv_w = p->conv_w; sa.conv_b = p->conv_b; sa.A = p->A; sa.D = p->D; sa.dt_bias = p->dt_bias;
                sa.c_rows = reinterpret_cast<const __bf16*>(ws + plan.off_crows[s]);
                sa.b_t = reinterpret_cast<const __bf16*>(ws + plan.off_bt[s]);
                sa.score_op = reinterpret_cast<const float*>(ws + plan.off_score[s]);
                sa.out = out->ptr; sa.out_sb = out->stride_batch; sa.out_st = out->stride_token;
                sa.partial = reinterpret_cast<float*>(ws + plan.off_partial);
                sa.h_in = (s == 0 && block_variant) ? h_in : nullptr;
                sa.h_out = (s == 0 && block_variant) ? h_out : nullptr;
                sa.tail_in = (s == 0 && block_variant) ? tail_in : nullptr;
                sa.L = d->seqlen; sa.Dn = d->d_inner; sa.H = d->n_heads; sa.HG = d->n_heads / d->n_groups;
                sa.G = d->n_groups; sa.K = d->d_conv; sa.tail_ch = tail_ch; sa.nchunk = plan.ssd_chunks;
                sa.parts = plan.ssd_parts; sa.part_chunks = plan.ssd_part_chunks;
                sa.part_subs = plan.ssd_part_subs; sa.sub_chunks = plan.ssd_sub_chunks;
                sa.part_state = reinterpret_cast<float*>(ws + plan.off_pstate[s]);
                sa.part_decay = reinterpret_cast<float*>(ws + plan.off_pdecay[s]);
                sa.dir = s == 0 ? 1 : -1;
                sa.mode = separate ? kSsdFinalOnly
                                   : s == 1 ? (raw ? kSsdPartialRaw : kSsdPartial) : (raw ? kSsdFinalAddRaw : kSsdFinalAdd);
                sa.out_ch_off = separate ? s * d->d_inner : 0;
                sa.dt_softplus = d->dt_softplus; sa.d_per_head = d->d_kind == BIMAMBA_D_PER_HEAD;
                // calls of several chunks that need no time parts walk sixteen waves wide (the row offsets of a chunk's
                // gate / output rows are 32-bit there) unless BIMAMBA_NO_WIDE is set
                constexpr int64_t kMaxWideStride = 1 << 24;
                sa.wide = plan.ssd_parts == 1 && plan.ssd_chunks >= 2 && in_f->z.stride_token <= kMaxWideStride &&
                          in_b->z.stride_token <= kMaxWideStride && out->stride_token <= kMaxWideStride &&
                          !getenv("BIMAMBA_NO_WIDE");
                return sa;
            };
            if (plan.ssd_parts > 1) {
                // time parts: every sub-part's end state from a zero start, then the states entering them
                SsdStatePair sp;
                SsdCarryArgs ca{};
                for (int s = 0; s < 2; s++) {
                    sp.dir[s] = scan_args(s);
                    ca.part_state[s] = sp.dir[s].part_state;
                    ca.part_decay[s] = sp.dir[s].part_decay;
                }
                launch_ssd_state(d->d_state, d->d_inner / d->n_heads, sp, plan.ssd_subs, d->batch, st);
                ca.h_in = block_variant ? h_in : nullptr;
                ca.batch = d->batch; ca.Dn = d->d_inner; ca.P = d->d_inner / d->n_heads; ca.H = d->n_heads;
                ca.parts = plan.ssd_subs;
                launch_ssd_carry(d->d_state, ca, st);
            }
            if (plan.ssd_chunks == 1) {
                SsdStatePair sp;
                for (int s = 0; s < 2; s++) sp.dir[s] = scan_args(s);
                launch_ssd_duo(d->d_state, d->d_inner / d->n_heads, sp, d->batch, st);
            } else {
                for (int s = 1; s >= 0; s--) launch_ssd_scan(d->d_state, d->d_inner / d->n_heads, scan_args(s), d->batch, st);
            }
            if (probe_stop) (void)hipEventRecord(probe_stop, st);
        } else {
        // 2. scan (summary + carry when the sequence is cut into segments) and combine
        SweepArgs sa{};
        for (int s = 0; s < 2; s++) {
            const bimamba_inputs* in = s == 0 ? in_f : in_b;
            const bimamba_params* p = s == 0 ? pf : pb;
            DirArgs& da = sa.dir[s];
            da.x = targ(in->x); da.z = targ(in->z); da.dt = targ(in->dt);
            da.bc = reinterpret_cast<const float*>(ws + plan.off_bc[s]);
            da.Braw = targ(in->B); da.Craw = targ(in->C);
            da.conv_w = p->conv_w; da.conv_b = p->conv_b; da.A = p->A; da.D = p->D; da.dt_bias = p->dt_bias;
        }
        sa.out = out->ptr; sa.out_sb = out->stride_batch; sa.out_st = out->stride_token;
        sa.partial = reinterpret_cast<float*>(ws + plan.off_partial);
        sa.h_in = block_variant ? h_in : nullptr;
        sa.h_out = block_variant ? h_out : nullptr;
        sa.tail_in = block_variant ? tail_in : nullptr;
        sa.carry = reinterpret_cast<float*>(ws + plan.off_carry);
        sa.sumdt = reinterpret_cast<float*>(ws + plan.off_sumdt);
        sa.L = d->seqlen; sa.Dn = d->d_inner; sa.P = d->d_inner / d->n_heads; sa.HG = d->n_heads / d->n_groups;
        sa.G = d->n_groups; sa.K = d->d_conv; sa.nseg = plan.nseg; sa.seg_len = plan.seg_len; sa.tail_ch = tail_ch;
        sa.dt_softplus = d->dt_softplus; sa.d_per_head = d->d_kind == BIMAMBA_D_PER_HEAD;
        sa.separate = d->combine == BIMAMBA_COMBINE_SEPARATE;
        sa.raw_partial = !sa.separate && same_tensor(in_f->z, in_b->z);
        sa.try_progression = 1;
        CarryArgs ca{};
        ca.carry = sa.carry; ca.sumdt = sa.sumdt; ca.A[0] = pf->A; ca.A[1] = pb->A;
        ca.h_in = sa.h_in; ca.h_out = sa.h_out;
        ca.batch = d->batch; ca.nseg = plan.nseg; ca.Dn = d->d_inner; ca.P = sa.P;
        launch_scan(d, plan.split, one_launch, sa, ca, st, probe_start, probe_stop);
        }
    } else if (block_variant && d->batch > 0 && h_out && h_out != h_in) {
        // empty block: the state passes through unchanged
        const size_t bytes = (size_t)d->batch * d->d_inner * d->d_state * sizeof(float);
        if (h_in) {
            (void)hipMemcpyAsync(h_out, h_in, bytes, hipMemcpyDeviceToDevice, st);
        } else {
            // a kernel rather than a memset node, so the call stays safe to capture into a HIP graph
            const long long n = (long long)d->batch * d->d_inner * d->d_state;
            hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, h_out, n);
        }
    }
    // 3. conv tail for the next block
    if (block_variant && tail_out && d->batch > 0 && d->d_conv > 1) {
        TailArgs ta{};
        ta.x = targ(in_f->x); ta.B = targ(in_f->B); ta.C = targ(in_f->C);
        ta.tail_in = tail_in; ta.tail_out = tail_out;
        ta.batch = d->batch; ta.L = d->seqlen; ta.K = d->d_conv; ta.Dn = d->d_inner; ta.GN = GN; ta.tail_ch = tail_ch;
        const long long total = (long long)d->batch * tail_ch;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (d->io_dtype == BIMAMBA_BF16) hipLaunchKernelGGL(tail_kernel<IoBF16>, grid, dim3(256), 0, st, ta);
        else hipLaunchKernelGGL(tail_kernel<IoF32>, grid, dim3(256), 0, st, ta);
    }
    const hipError_t now = hipPeekAtLastError();
    return now == hipSuccess || now == pending ? BIMAMBA_OK : BIMAMBA_ERR_HIP;
}

constexpr int kMaxScratchDevices = 64;
std::atomic<void*> g_scratch_addr[kMaxScratchDevices];   // per device: each GPU holds its own copy of the array

// The current device's copy of `scratch`, asked once per device with that device current.
int static_scratch(void** addr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxScratchDevices) return BIMAMBA_ERR_HIP;
    void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BIMAMBA_ERR_HIP;
        g_scratch_addr[dev].store(p, std::memory_order_release);
    }
    *addr = p;
    return BIMAMBA_OK;
}

}  // namespace

extern "C" {

int bimamba_fwd(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                const bimamba_inputs* in_f, const bimamba_inputs* in_b, const bimamba_tensor* out, void* workspace,
                size_t workspace_bytes, void* hip_stream)
{
    return run(desc, pf, pb, in_f, in_b, nullptr, nullptr, nullptr, nullptr, out, workspace, workspace_bytes, hip_stream,
               false);
}

int bimamba_block_fwd(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                      const bimamba_inputs* in_f, const bimamba_inputs* in_b, const float* h_in, const void* tail_in,
                      float* h_out, void* tail_out, const bimamba_tensor* out, void* workspace, size_t workspace_bytes,
                      void* hip_stream)
{
    return run(desc, pf, pb, in_f, in_b, h_in, tail_in, h_out, tail_out, out, workspace, workspace_bytes, hip_stream,
               true);
}

int bimamba_block_fwd_static(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                             const bimamba_inputs* in_f, const bimamba_inputs* in_b, const float* h_in,
                             const void* tail_in, float* h_out, void* tail_out, const bimamba_tensor* out,
                             void* hip_stream)
{
    int rc = check_desc(desc);
    if (rc) return rc;
    if (make_plan(desc, false).total > (size_t)BIMAMBA_STATIC_SCRATCH_BYTES) return BIMAMBA_ERR_SCRATCH_EXCEEDED;
    void* ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    return run(desc, pf, pb, in_f, in_b, h_in, tail_in, h_out, tail_out, out, ws, BIMAMBA_STATIC_SCRATCH_BYTES, hip_stream,
               true);
}

// ---- gradients -------------------------------------------------------------------------------------------------
namespace {
struct BwdPlan {
    bool dense;   // the two-waves-per-SIMD form of the kernels (shorter chunks for 16 states)
    int chunk, nchunk;
    int tiles_per_group;
    size_t off_bc[2], off_state, off_parked, off_part[2], total;
};

int check_bwd_desc(const bimamba_desc* d)
{
    const int rc = check_desc(d);
    if (rc) return rc;
    if (d->n_heads != d->d_inner || d->a_kind != BIMAMBA_A_PER_HEAD_STATE || d->d_kind != BIMAMBA_D_PER_CHANNEL ||
        d->conv_bc || !bm::bwd_supported(d->d_state))
        return BIMAMBA_ERR_UNSUPPORTED;
    return BIMAMBA_OK;
}

BwdPlan make_bwd_plan(const bimamba_desc* d)
{
    BwdPlan p{};
    p.dense = bm::bwd_dense(d->d_inner, d->batch);
    p.chunk = bm::bwd_chunk_tokens(d->d_state, p.dense);
    p.nchunk = d->seqlen > 0 ? (d->seqlen + p.chunk - 1) / p.chunk : 1;
    const size_t bc = align_up((size_t)d->batch * d->seqlen * d->n_groups * 2 * d->d_state * sizeof(float), 256);
    const size_t parked = align_up((size_t)d->batch * d->seqlen * d->d_inner * sizeof(Parked), 256);
    size_t off = 0;
    p.off_bc[0] = off; off += bc;
    p.off_bc[1] = off; off += bc;    // sized for separate activations
    p.off_state = off; off += align_up((size_t)2 * d->batch * p.nchunk * d->d_inner * d->d_state * sizeof(float), 256);
    p.off_parked = off; off += parked;
    // per-wave partial sums of dB | dC: one slot per channel tile of a group and direction
    p.tiles_per_group = (d->d_inner / d->n_groups + 63) / 64;
    const size_t part = align_up((size_t)d->batch * d->seqlen * d->n_groups * p.tiles_per_group * 2 * d->d_state * sizeof(float), 256);
    p.off_part[0] = off; off += part;
    p.off_part[1] = off; off += part;
    p.total = off;
    return p;
}
}  // namespace

int bimamba_bwd(const bimamba_desc* d, const bimamba_params* pf, const bimamba_params* pb, const bimamba_inputs* in_f,
                const bimamba_inputs* in_b, const bimamba_tensor* dout, const bimamba_input_grads* din_f,
                const bimamba_input_grads* din_b, const bimamba_param_grads* dpf, const bimamba_param_grads* dpb,
                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int rc = check_bwd_desc(d);
    if (rc) return rc;
    const size_t elem = d->io_dtype == BIMAMBA_BF16 ? 2 : 4;
    if ((rc = check_params(pf))) return rc;
    if ((rc = check_params(pb))) return rc;
    if (!in_f || !dout || !din_f || !dpf || !dpb) return BIMAMBA_ERR_NULL_POINTER;
    if (!in_b) in_b = in_f;
    if ((rc = check_inputs(in_f, d, elem))) return rc;
    if ((rc = check_inputs(in_b, d, elem))) return rc;
    const bool shared = same_inputs(in_f, in_b);
    if (shared ? din_b != nullptr && din_b != din_f : din_b == nullptr) return BIMAMBA_ERR_NULL_POINTER;
    if (shared) din_b = nullptr;
    const int out_ch = d->combine == BIMAMBA_COMBINE_SEPARATE ? 2 * d->d_inner : d->d_inner;
    if ((rc = check_tensor(*dout, out_ch, elem, d))) return rc;
    const bool live = d->batch > 0 && d->seqlen > 0;
    for (const bimamba_input_grads* g : {din_f, din_b}) {
        if (!g) continue;
        if ((rc = check_tensor(g->dx, d->d_inner, elem, d))) return rc;
        if ((rc = check_tensor(g->dz, d->d_inner, elem, d))) return rc;
        if ((rc = check_tensor(g->ddt, d->n_heads, elem, d))) return rc;
        if (live && (!g->dB || !g->dC)) return BIMAMBA_ERR_NULL_POINTER;
        if (!is_aligned(g->dB, 4) || !is_aligned(g->dC, 4)) return BIMAMBA_ERR_MISALIGNED;
    }
    if (dpf == dpb) return BIMAMBA_ERR_ALIAS;
    for (const bimamba_param_grads* g : {dpf, dpb}) {
        if (!g->dconv_w || !g->dA || !g->dD) return BIMAMBA_ERR_NULL_POINTER;
        if (!is_aligned(g->dconv_w, 4) || !is_aligned(g->dA, 4) || !is_aligned(g->dD, 4) || !is_aligned(g->dconv_b, 4) ||
            !is_aligned(g->ddt_bias, 4))
            return BIMAMBA_ERR_MISALIGNED;
    }
    const BwdPlan plan = make_bwd_plan(d);
    if (!workspace) return BIMAMBA_ERR_NULL_POINTER;
    if (!is_aligned(workspace, 16)) return BIMAMBA_ERR_MISALIGNED;
    if (workspace_bytes < plan.total) return BIMAMBA_ERR_WORKSPACE_TOO_SMALL;

    const hipError_t pending = hipPeekAtLastError();
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int GN = d->n_groups * d->d_state;
    const bool bf16 = d->io_dtype == BIMAMBA_BF16;

    // parameter gradients are sums over the batch: zero them even for an empty call
    for (const bimamba_param_grads* g : {dpf, dpb}) {
        bm::launch_bwd_zero(g->dconv_w, (long long)d->d_inner * d->d_conv, st);
        bm::launch_bwd_zero(g->dconv_b, d->d_inner, st);
        bm::launch_bwd_zero(g->dA, (long long)d->d_inner * d->d_state, st);
        bm::launch_bwd_zero(g->dD, d->d_inner, st);
        bm::launch_bwd_zero(g->ddt_bias, d->d_inner, st);
    }
    if (live) {
        const int nbuf = shared ? 1 : 2;
        for (int s = 0; s < nbuf; s++) {
            const bimamba_inputs* in = s == 0 ? in_f : in_b;
            PrepArgs pa{};
            pa.B = targ(in->B);
            pa.C = targ(in->C);
            pa.dst = reinterpret_cast<float*>(ws + plan.off_bc[s]);
            pa.batch = d->batch; pa.L = d->seqlen; pa.G = d->n_groups; pa.N = d->d_state; pa.K = d->d_conv;
            pa.Dn = d->d_inner; pa.tail_ch = d->d_inner; pa.conv_bc = 0; pa.dir = s == 0 ? 1 : -1;
            const long long total = (long long)d->batch * d->seqlen * 2 * GN;
            const dim3 grid((unsigned)((total + 255) / 256));
            if (bf16) hipLaunchKernelGGL(prep_bc_kernel<IoBF16>, grid, dim3(256), 0, st, pa);
            else hipLaunchKernelGGL(prep_bc_kernel<IoF32>, grid, dim3(256), 0, st, pa);
        }
        BwdArgs a{};
        for (int s = 0; s < 2; s++) {
            const bimamba_inputs* in = s == 0 ? in_f : in_b;
            const bimamba_params* p = s == 0 ? pf : pb;
            const bimamba_param_grads* g = s == 0 ? dpf : dpb;
            const bimamba_input_grads* gi = (s == 0 || !din_b) ? din_f : din_b;
            DirArgs& da = a.dir[s];
            da.x = targ(in->x); da.z = targ(in->z); da.dt = targ(in->dt);
            da.bc = reinterpret_cast<const float*>(ws + plan.off_bc[shared ? 0 : s]);
            da.conv_w = p->conv_w; da.conv_b = p->conv_b; da.A = p->A; da.D = p->D; da.dt_bias = p->dt_bias;
            // shared activations: both directions' waves fill slots of one buffer (the two parts are adjacent)
            a.bc_part[s] = reinterpret_cast<float*>(ws + plan.off_part[shared ? 0 : s]);
            a.gdx[s] = targ(gi->dx); a.gdz[s] = targ(gi->dz); a.gddt[s] = targ(gi->ddt);
            a.dA[s] = g->dA; a.dD[s] = g->dD; a.dconv_w[s] = g->dconv_w; a.dconv_b[s] = g->dconv_b; a.ddt_bias[s] = g->ddt_bias;
        }
        a.dout = targ(*dout);
        a.state = reinterpret_cast<float*>(ws + plan.off_state);
        a.parked = reinterpret_cast<Parked*>(ws + plan.off_parked);
        a.L = d->seqlen; a.Dn = d->d_inner; a.G = d->n_groups; a.K = d->d_conv; a.nchunk = plan.nchunk;
        a.dt_softplus = d->dt_softplus; a.separate = d->combine == BIMAMBA_COMBINE_SEPARATE;
        a.park = shared;
        a.bc_slots = plan.tiles_per_group * (shared ? 2 : 1);
        a.bc_slot_of_rev = shared ? plan.tiles_per_group : 0;
        bm::launch_bwd(d->d_state, bf16, plan.dense, a, d->batch, st);
        for (int s = 0; s < (shared ? 1 : 2); s++) {
            const bimamba_input_grads* gi = s == 0 ? din_f : din_b;
            BwdBcArgs ba{};
            ba.part = a.bc_part[s];
            ba.dB = gi->dB; ba.dC = gi->dC;
            ba.rows = (long long)d->batch * d->seqlen * d->n_groups;
            ba.slots = a.bc_slots; ba.N = d->d_state;
            bm::launch_bwd_bc(ba, st);
        }
    }
    const hipError_t now = hipPeekAtLastError();
    return (now == hipSuccess || now == pending) ? BIMAMBA_OK : BIMAMBA_ERR_HIP;
}

size_t bimamba_bwd_workspace_bytes(const bimamba_desc* desc)
{
    if (check_bwd_desc(desc)) return 0;
    return make_bwd_plan(desc).total;
}

size_t bimamba_workspace_bytes(const bimamba_desc* desc, int block_variant)
{
    (void)block_variant;
    if (check_desc(desc)) return 0;
    // sized for the larger case (the two directions reading different activations)
    return make_plan(desc, false).total;
}

int bimamba_time_chunks(const bimamba_desc* desc)
{
    if (check_desc(desc)) return 0;
    const Plan p = make_plan(desc, true);
    return p.ssd ? p.ssd_parts : p.nseg;
}

void bimamba_profile_next_call(void* ev_start, void* ev_stop)
{
    g_probe_start = reinterpret_cast<hipEvent_t>(ev_start);
    g_probe_stop = reinterpret_cast<hipEvent_t>(ev_stop);
}

const char* bimamba_status_string(int status)
{
    switch (status) {
        case BIMAMBA_OK: return "ok";
        case BIMAMBA_ERR_NULL_POINTER: return "a required pointer is NULL";
        case BIMAMBA_ERR_BAD_SHAPE: return "bad shape: non-positive or inconsistent dimension or stride";
        case BIMAMBA_ERR_UNSUPPORTED: return "unsupported dtype, d_state, d_conv, grouping or token stride";
        case BIMAMBA_ERR_MISALIGNED: return "misaligned pointer";
        case BIMAMBA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case BIMAMBA_ERR_HIP: return "HIP launch error";
        case BIMAMBA_ERR_ALIAS: return "the output overlaps an input";
        case BIMAMBA_ERR_SCRATCH_EXCEEDED: return "the call needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

int bimamba_version(void) { return BIMAMBA_VERSION; }

}  // extern "C"
