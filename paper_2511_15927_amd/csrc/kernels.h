// Device code of the bidirectional Mamba mixer path for gfx950 (CDNA4, wave64).
//
// Mapping.  A chain is one (direction, batch element, channel): it walks the sequence token by token with its
// d_state recurrence values in registers.  S adjacent lanes share a chain, each holding d_state/S of the states
// (S = 1, 2 or 4, chosen by the host so that the launch has enough waves to fill 1024 SIMDs); their partial dot
// products C_t . h_t are summed with DPP lane swaps.  A wave therefore covers 64/S adjacent channels and every
// per-token access of x / dt / z / out is one contiguous run, addressed as a wave-uniform row plus a constant lane
// offset.  A workgroup holds the forward wave and the reverse wave of two adjacent channel tiles, one wave for each of
// a CU's four SIMDs.  For the additive combine (eq. 6) the two waves of a tile meet in the middle of the segment: in
// the first half of its walk each wave parks its output as an fp32 partial, in the second half it adds the partial
// the other wave parked there and performs the single rounding to the I/O dtype.
//
// With up to 16 states split over several lanes, those lanes also deal the tokens among themselves: lane j of a chain
// owns token j of every group of S tokens and does that token's per-channel work (loads, conv, SiLUs, gate, store)
// alone, the others reading what they need of it through lane-permute operands (run_tiles_dealt).
//
// B_t and C_t come from an fp32 copy made by prep_bc_kernel.  With S = 1 they are wave-uniform and are fetched one
// token ahead with scalar loads; with S > 1 each lane needs its own slice, so a tile of rows is staged through LDS
// (private to the wave, no barrier) and read back one token ahead.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace bm {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Read-only for the whole kernel and wave-uniform: the constant address space lets the compiler fetch it with
// scalar loads even when unrelated global stores sit between the loads.
typedef const __attribute__((address_space(4))) float* uniform_ro_ptr;

struct TensorArg {
    const void* p;
    long long sb, st;  // batch / token stride in elements
};

struct DirArgs {
    TensorArg x, z, dt;
    const float* bc;  // prepared fp32 B|C rows: [batch][L][G][2N]
    TensorArg Braw, Craw;  // the caller's B and C tensors (read directly by the short-call variant)
    const float* conv_w;
    const float* conv_b;
    const float* A;
    const float* D;
    const float* dt_bias;
};

struct SweepArgs {
    DirArgs dir[2];
    void* out;
    long long out_sb, out_st;
    float* partial;       // [batch][L][Dn] fp32 (ADD only)
    const float* h_in;    // [batch][Dn][N] or null
    float* h_out;         // or null; written by the sweep only when nseg == 1
    const void* tail_in;  // io dtype [batch][K-1][tail_ch] or null
    float* carry;         // [2][batch][nseg][Dn][N]: segment end states (summary) then segment start states (carry)
    float* sumdt;         // [2][batch][nseg][Dn]
    int L, Dn, P, HG, G, K, nseg, seg_len, tail_ch;
    int dt_softplus, d_per_head, separate;
    int raw_partial;      // both directions gate with the same z: park y ungated and gate once at the final store
    int try_progression;  // let each wave test whether its chains' A rows are arithmetic in n (see sweep_kernel)
    int layer_wgs;        // workgroups the dispatcher places before a CU gets its next one (the CU count); set by the launcher
    int turn_mask;        // 0: leave wave priorities alone; 1 / 3: two / up to four waves share a SIMD and take turns
};

// Buffer resource of a raw (untyped, unstrided) range starting at a wave-uniform address.  An access adds a
// wave-uniform byte offset and a 32-bit per-lane byte offset to that address inside the memory instruction itself, so
// it needs no vector address arithmetic.  The range is left unbounded: callers keep every offset inside the tensor.
typedef __amdgpu_buffer_rsrc_t Rsrc;
__device__ __forceinline__ Rsrc raw_range(const void* base)
{
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, -1, 0x00020000);
}

struct IoF32 {
    using T = float;
    static __device__ __forceinline__ float ld(const T* p) { return *p; }
    static __device__ __forceinline__ float cvt(T v) { return v; }
    static __device__ __forceinline__ void st(T* p, float v) { *p = v; }
    static __device__ __forceinline__ T ld_raw(Rsrc r, unsigned lane_off, int row_off)
    {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, lane_off, row_off, 0));
    }
    static __device__ __forceinline__ void st_raw(Rsrc r, unsigned lane_off, int row_off, float v)
    {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, lane_off, row_off, 0);
    }
};
struct IoBF16 {
    using T = unsigned short;
    static __device__ __forceinline__ float cvt(T v) { return __uint_as_float(((unsigned)v) << 16); }
    static __device__ __forceinline__ float ld(const T* p) { return cvt(*p); }
    static __device__ __forceinline__ T round(float v)
    {
        __bf16 r = (__bf16)v;  // round to nearest even (v_cvt_pk_bf16_f32)
        return __builtin_bit_cast(unsigned short, r);
    }
    static __device__ __forceinline__ void st(T* p, float v) { *p = round(v); }
    static __device__ __forceinline__ T ld_raw(Rsrc r, unsigned lane_off, int row_off)
    {
        return __builtin_amdgcn_raw_buffer_load_b16(r, lane_off, row_off, 0);
    }
    static __device__ __forceinline__ void st_raw(Rsrc r, unsigned lane_off, int row_off, float v)
    {
        __builtin_amdgcn_raw_buffer_store_b16(round(v), r, lane_off, row_off, 0);
    }
};

// A result in the I/O dtype (one rounding to nearest even for bf16).
template <typename IO>
__device__ __forceinline__ typename IO::T io_value(float v)
{
    if constexpr (sizeof(typename IO::T) == 2) return IO::round(v);
    else return v;
}

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float silu(float v) { return v * __builtin_amdgcn_rcpf(1.0f + fast_exp2(-kLog2e * v)); }
// softplus(v) = max(v, 0) + log1p(e), e = exp(-|v|) in (0, 1].  log1p(e) is taken as log(w) * e / (w - 1) with
// w = fl(1 + e), which cancels the rounding of the sum and keeps full relative accuracy for small e.
__device__ __forceinline__ float softplus(float v)
{
    const float e = fast_exp2(-kLog2e * fabsf(v));
    const float w = 1.0f + e;
    const float d = w - 1.0f;
    const float l = d == 0.0f ? e : (__builtin_amdgcn_logf(w) * kLn2) * e * __builtin_amdgcn_rcpf(d);
    return fmaxf(v, 0.0f) + l;
}

// Sum over the S adjacent lanes of a chain (S = 1, 2, 4); every lane ends up with the total.
template <int S>
__device__ __forceinline__ float sum_over_chain_lanes(float v)
{
    if (S >= 2) {  // quad_perm [1,0,3,2]
        const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true);
        v += __int_as_float(o);
    }
    if (S >= 4) {  // quad_perm [2,3,0,1]
        const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true);
        v += __int_as_float(o);
    }
    return v;
}

// The value lane J of the caller's chain holds (S = 2: lane pairs, S = 4: quads), by a quad-permute move.
template <int S, int J>
__device__ __forceinline__ float chain_lane_value(float v)
{
    static_assert((S == 2 || S == 4) && J < S, "chains are lane pairs or quads");
    constexpr int kSel = S == 2 ? (J == 0 ? 0xA0 : 0xF5) : J * 0x55;  // [0,0,2,2] / [1,1,3,3]; [J,J,J,J]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kSel, 0xF, 0xF, true));
}

enum { kSweep = 0, kSummary = 1 };
// Where a token's B|C row comes from: the fp32 rows prep_bc_kernel prepared, or (short calls, one lane per chain, no
// conv on B and C) a copy of the caller's rows that each wave converts into LDS itself at kernel start, which saves
// the preparation launch when a call is a few dozen tokens long.
enum { kBcPrepared = 0, kBcStaged = 1 };
constexpr int kShortCallTokens = 64;
// How the decay exp(Delta A[h, n]) is formed: one exponential per state; one per token for a scalar A per head; or, when
// A is an arithmetic progression in n (detected on the device), two exponentials per token, a_n = a_first r^n.
enum { kAPerState = 0, kAScalar = 1, kAProgression = 2 };
// What a range of the walk does with its result:
//   Partial      park g = y * SiLU(z)           PartialRaw   park y (gate later)
//   FinalAdd     store g + partial              FinalAddRaw  store (y + partial) * SiLU(z)
//   FinalOnly    store g (separate halves)      NoOutput     state only (segment summary)
enum { kModePartial = 0, kModeFinalAdd = 1, kModeFinalOnly = 2, kModeNoOutput = 3, kModePartialRaw = 4, kModeFinalAddRaw = 5 };
__host__ __device__ constexpr bool mode_reads_z(int m) { return m != kModeNoOutput && m != kModePartialRaw; }
__host__ __device__ constexpr bool mode_reads_partial(int m) { return m == kModeFinalAdd || m == kModeFinalAddRaw; }

// TILE (template parameter below): tokens whose loads are in flight while the previous tile is being computed.  8 when
// a SIMD holds one or two waves (the prefetch depth hides HBM latency); 4 when it can hold four or more (fewer
// registers per wave, and the other waves hide the latency).

// TILE consecutive tokens (scan order) of one tensor as a raw range: the range starts at the tile's lowest-address
// row, so a token's row offset is never negative whatever the sign of the caller's stride or the direction of the
// walk.  first / inc are bytes; |inc| * (TILE - 1) fits an int (the host rejects larger token strides).
template <int TILE>
struct TileRows {
    Rsrc range;
    int first, inc;  // row offset of the tile's first token, signed step per token
    __device__ __forceinline__ int row(int i) const { return first + i * inc; }
};

template <int TILE, typename T>
__device__ __forceinline__ TileRows<TILE> tile_rows(T* first_row, long long step)
{
    TileRows<TILE> t;
    t.inc = (int)step * (int)sizeof(T);
    // Row offsets are cheap to form (one scalar add each); left visible as loop invariants they would all be kept live
    // across the walk, a few dozen scalar registers more than there are.
    asm volatile("" : "+s"(t.inc));
    t.first = step < 0 ? -(TILE - 1) * t.inc : 0;
    t.range = raw_range(step < 0 ? first_row + (TILE - 1) * step : first_row);
    return t;
}

// The lane's element of a row given by pointer (tokens outside whole tiles).
template <typename T>
__device__ __forceinline__ T* lane_elem(T* row, unsigned byte_off)
{
    using Byte = std::conditional_t<std::is_const_v<T>, const char, char>;
    return reinterpret_cast<T*>(reinterpret_cast<Byte*>(row) + byte_off);
}

// Per-lane constants and running state of one chain slice.  Row pointers are wave-uniform and advance by signed
// per-token steps; the lane's place in a row is a constant byte offset.
template <int N, int S, int AKIND, typename IO>
struct Chain {
    using T = typename IO::T;
    static constexpr int NS = N / S;
    float h[NS];
    float a2[AKIND == kAPerState ? NS : 1];  // A * log2(e) (kAProgression: of the slice's first state)
    float d2;                       // kAProgression: (A[h,1] - A[h,0]) * log2(e)
    float w4[4];                    // conv taps, w4[3] on the current token
    float cb, dval, dtb, sum_dt;
    float xh[3];                    // previous raw x, xh[0] most recent
    const T *xrow, *zrow, *dtrow;
    T* orow;
    float* prow;
    const float* bcrow;             // this token's B|C row of the tile's group
    long long xs, zs, dts, os, ps, bcs;
    unsigned ch_io, head_io, ch_f32;  // the lane's byte offset into a row: channel / head in the I/O dtype, channel in fp32
    unsigned sub;                   // slice index (lane % S)
    int tok, tstep;                 // kBcStaged: current token and its signed step (rows are indexed by token in LDS)
};

template <typename IO, int TILE>
struct RawTile {
    typename IO::T x[TILE], z[TILE], dt[TILE];
    float part[TILE];
};

template <int N, int S, int AKIND, typename IO, int MODE, int TILE>
__device__ __forceinline__ void load_tile(const Chain<N, S, AKIND, IO>& c, long long ahead, RawTile<IO, TILE>& r)
{
    const TileRows<TILE> tx = tile_rows<TILE>(c.xrow + ahead * c.xs, c.xs);
    const TileRows<TILE> td = tile_rows<TILE>(c.dtrow + ahead * c.dts, c.dts);
    const TileRows<TILE> tz = tile_rows<TILE>(c.zrow + ahead * c.zs, c.zs);
    const TileRows<TILE> tp = tile_rows<TILE>(c.prow + ahead * c.ps, c.ps);
#pragma unroll
    for (int i = 0; i < TILE; i++) {
        r.x[i] = IO::ld_raw(tx.range, c.ch_io, tx.row(i));
        r.dt[i] = IO::ld_raw(td.range, c.head_io, td.row(i));
        if (mode_reads_z(MODE)) r.z[i] = IO::ld_raw(tz.range, c.ch_io, tz.row(i));
        if (mode_reads_partial(MODE)) r.part[i] = IoF32::ld_raw(tp.range, c.ch_f32, tp.row(i));
    }
}

// Where a token's result goes: token i of a tile addressed as raw ranges, or rows given by pointer.
template <typename IO, int TILE>
struct TileSink {
    const TileRows<TILE>&o, &p;
    unsigned ch_io, ch_f32;
    int i;
    __device__ __forceinline__ void park(float v) const { IoF32::st_raw(p.range, ch_f32, p.row(i), v); }
    __device__ __forceinline__ void final(float v) const { IO::st_raw(o.range, ch_io, o.row(i), v); }
};
template <typename IO>
struct RowSink {
    typename IO::T* orow;
    float* prow;
    unsigned ch_io, ch_f32;
    __device__ __forceinline__ void park(float v) const { *lane_elem(prow, ch_f32) = v; }
    __device__ __forceinline__ void final(float v) const { IO::st(lane_elem(orow, ch_io), v); }
};

// One token's B (first NS) and C (last NS) values for this lane's state slice.
template <int NS>
struct BcRow {
    float v[2 * NS];
};

// S = 1 rows of up to 16 states are fetched one token ahead into scalar registers; longer rows are read where used.
template <int N, int S>
constexpr bool kBcScalarAhead = (S == 1 && N <= 16);

template <int N>
__device__ __forceinline__ void load_bc_scalar(const float* p, BcRow<N>& r)
{
    uniform_ro_ptr q = (uniform_ro_ptr)p;
#pragma unroll
    for (int n = 0; n < 2 * N; n++) r.v[n] = q[n];
}

// Lane-private slice straight from global memory (tokens outside whole tiles).
template <int N, int S>
__device__ __forceinline__ void load_bc_direct(const float* row, unsigned sub, BcRow<N / S>& r)
{
    constexpr int NS = N / S;
    const float4* b4 = reinterpret_cast<const float4*>(row + sub * NS);
    const float4* c4 = reinterpret_cast<const float4*>(row + N + sub * NS);
#pragma unroll
    for (int j = 0; j < NS / 4; j++) {
        const float4 bv = b4[j], cv = c4[j];
        r.v[4 * j] = bv.x; r.v[4 * j + 1] = bv.y; r.v[4 * j + 2] = bv.z; r.v[4 * j + 3] = bv.w;
        r.v[NS + 4 * j] = cv.x; r.v[NS + 4 * j + 1] = cv.y; r.v[NS + 4 * j + 2] = cv.z; r.v[NS + 4 * j + 3] = cv.w;
    }
}

// Lane-private slice of token i of a staged tile in LDS ([TILE][2N] floats).
template <int N, int S>
__device__ __forceinline__ void load_bc_lds(const float* tile, int i, unsigned sub, BcRow<N / S>& r)
{
    load_bc_direct<N, S>(tile + i * 2 * N, sub, r);
}

// One token of one chain slice: conv + SiLU, discretise, state updates, skip term, gate, output.  Advances the B|C
// row and the token counter; the caller advances the other rows.
// REFILL (scalar-register rows): `row` holds this token's B|C on entry and the values at `next` on exit.  The
// state updates (which read B) and the output dot product (which reads C) run as two loops, and each half of the row
// is requested again as soon as its loop is done, into the registers it just freed: one row of scalar registers
// instead of two, with more than half a token of work between a request and its first use.
template <int N, int S, int AKIND, typename IO, int MODE, bool REFILL, typename Sink>
__device__ __forceinline__ void token_step(Chain<N, S, AKIND, IO>& c, typename IO::T xraw, float delta,
                                           typename IO::T zraw, float part, BcRow<N / S>& row, const float* next,
                                           const Sink& sink)
{
    constexpr int NS = N / S;
    const float x0 = IO::cvt(xraw);
    float pre = c.cb;
    pre = fmaf(c.w4[0], c.xh[2], pre);
    pre = fmaf(c.w4[1], c.xh[1], pre);
    pre = fmaf(c.w4[2], c.xh[0], pre);
    pre = fmaf(c.w4[3], x0, pre);
    c.xh[2] = c.xh[1];
    c.xh[1] = c.xh[0];
    c.xh[0] = x0;
    // With several lanes per chain the conv SiLU and the gate SiLU of a token are evaluated in one pass: slice 0 of the
    // chain feeds the conv pre-activation, slice 1 feeds z, and both results are handed to all lanes of the chain with
    // quad-permute moves (the values are the ones every lane would have computed for itself).
    constexpr bool kSharedSilu = S >= 2 && MODE != kModeNoOutput && MODE != kModePartialRaw;
    float xc, zg = 0.0f;
    if constexpr (kSharedSilu) {
        const float sv = silu(c.sub == 1 ? IO::cvt(zraw) : pre);
        xc = chain_lane_value<S, 0>(sv);
        zg = chain_lane_value<S, 1>(sv);
    } else {
        xc = silu(pre);
        if constexpr (MODE != kModeNoOutput && MODE != kModePartialRaw) zg = silu(IO::cvt(zraw));
    }
    const float u = delta * xc;
    float y = 0.0f;
    uniform_ro_ptr bcmem = (uniform_ro_ptr)c.bcrow;  // only for S = 1 rows too long to prefetch
    constexpr bool kFromMem = (S == 1 && N > 16);
    auto bc = [&](int n) -> float { return kFromMem ? bcmem[n < NS ? n : n - NS + N] : row.v[n]; };
    if constexpr (REFILL) {
        uniform_ro_ptr q = (uniform_ro_ptr)next;
        if (AKIND == kAPerState) {
#pragma unroll
            for (int n = 0; n < NS; n++) c.h[n] = fmaf(fast_exp2(delta * c.a2[n]), c.h[n], u * row.v[n]);
        } else if (AKIND == kAProgression) {
            float an = fast_exp2(delta * c.a2[0]);
            const float ratio = fast_exp2(delta * c.d2);
#pragma unroll
            for (int n = 0; n < NS; n++) {
                c.h[n] = fmaf(an, c.h[n], u * row.v[n]);
                an *= ratio;
            }
        } else {
            const float a = fast_exp2(delta * c.a2[0]);
#pragma unroll
            for (int n = 0; n < NS; n++) c.h[n] = fmaf(a, c.h[n], u * row.v[n]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NS; n++) row.v[n] = q[n];
        __builtin_amdgcn_sched_barrier(0);
        if (MODE != kModeNoOutput) {
#pragma unroll
            for (int n = 0; n < NS; n++) y = fmaf(row.v[NS + n], c.h[n], y);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int n = 0; n < NS; n++) row.v[NS + n] = q[N + n];
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (AKIND == kAPerState) {
#pragma unroll
        for (int n = 0; n < NS; n++) {
            const float a = fast_exp2(delta * c.a2[n]);
            c.h[n] = fmaf(a, c.h[n], u * bc(n));
            if (MODE != kModeNoOutput) y = fmaf(bc(NS + n), c.h[n], y);
        }
    } else if (AKIND == kAProgression) {
        float an = fast_exp2(delta * c.a2[0]);
        const float ratio = fast_exp2(delta * c.d2);
#pragma unroll
        for (int n = 0; n < NS; n++) {
            c.h[n] = fmaf(an, c.h[n], u * bc(n));
            if (MODE != kModeNoOutput) y = fmaf(bc(NS + n), c.h[n], y);
            an *= ratio;
        }
    } else {
        const float a = fast_exp2(delta * c.a2[0]);
#pragma unroll
        for (int n = 0; n < NS; n++) {
            c.h[n] = fmaf(a, c.h[n], u * bc(n));
            if (MODE != kModeNoOutput) y = fmaf(bc(NS + n), c.h[n], y);
        }
    }
    if (MODE == kModeNoOutput) {
        c.sum_dt += delta;
    } else {
        y = sum_over_chain_lanes<S>(y);
        y = fmaf(c.dval, xc, y);
        if (MODE == kModePartialRaw) {
            sink.park(y);
        } else if (MODE == kModeFinalAddRaw) {
            sink.final((y + part) * zg);
        } else {
            const float g = y * zg;
            if (MODE == kModePartial) sink.park(g);
            else sink.final(MODE == kModeFinalAdd ? g + part : g);
        }
    }
    c.bcrow += c.bcs;
    c.tok += c.tstep;
}

template <int N, int S, int AKIND, typename IO>
__device__ __forceinline__ void advance_rows(Chain<N, S, AKIND, IO>& c, int tokens)
{
    c.xrow += tokens * c.xs;
    c.dtrow += tokens * c.dts;
    c.zrow += tokens * c.zs;
    c.orow += tokens * c.os;
    c.prow += tokens * c.ps;
}

// Waves that share a SIMD take turns at the top issue priority.  Left alone, the arbiter favours the oldest wave: the
// workgroups a CU received first run ahead, finish early and leave the younger ones alone on the SIMD, where a
// single wave cannot keep the vector pipe busy (measured at two waves per SIMD: lifetimes 1.84 and 2.38 ms for the two
// halves of the launch, 2.27 ms for all with turns).  The turn is a function of the constant-rate clock, which all
// waves read alike, and of the order in which the workgroups reached the CU, so at any moment the waves of a SIMD
// hold different priorities however far they have drifted apart.
constexpr int kTurnShift = 12;  // a turn lasts 2^12 ticks of the 100 MHz clock
__device__ __forceinline__ void take_turn(const SweepArgs& a)
{
    // read from the kernel arguments where needed, not carried through the walk in registers
    const unsigned mask = (unsigned)a.turn_mask;
    if (mask == 0) return;
    const unsigned turn = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) / (unsigned)a.layer_wgs;
    const unsigned p = ((unsigned)(wall_clock64() >> kTurnShift) + turn) & mask;
    if (p == 0) __builtin_amdgcn_s_setprio(0);
    else if (p == 1) __builtin_amdgcn_s_setprio(1);
    else if (p == 2) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(3);
}

// ---- Dealt tokens (S = 2 or 4 lanes per chain) -----------------------------------------------------------------
// The S lanes of a chain split its states, and they also split the per-channel work of S consecutive tokens (a
// group): lane j of the chain OWNS token j of every group.  Only the owner loads that token's x, Delta, z and partial,
// converts them, evaluates the conv, both SiLUs and the softplus, forms u = Delta * xc and the decay ratio, and later
// finishes and stores the token's result.  What the other lanes need of a token (Delta, u, the ratio) they read from
// the owner's registers through the quad-permute operand of the consuming instruction.  Per lane and token that leaves
// the 4 * N/S state instructions, one exponential and the reduction; everything else is paid once per group instead
// of once per token, and a wave issues one load or store instruction per group and tensor instead of one per token.
//
// The conv window of token i reaches back to tokens i-1 .. i-3, which other lanes own: token i-k sits in lane
// (j - k) mod S, in the same group when k <= j and ceil((k - j) / S) groups back otherwise.  Each lane keeps its own raw
// x of the last few groups and holds, per (k, groups back), either the tap weight or zero, so the window is a fixed
// sequence of multiply-adds on lane-rotated values with no selects.  (A zero weight multiplies a token the window does
// not contain; with finite inputs that adds nothing.)
template <int S>
__host__ __device__ constexpr int dealt_groups_back(int j, int k) { return k <= j ? 0 : (k - j + S - 1) / S; }
template <int S>
__host__ __device__ constexpr bool dealt_term_exists(int k, int d)
{
    for (int j = 0; j < S; j++)
        if (dealt_groups_back<S>(j, k) == d) return true;
    return false;
}

// The value lane (own - k) mod S of the caller's chain holds.  k is a constant wherever this is called from an
// unrolled loop, so one move remains.
template <int S>
__device__ __forceinline__ float chain_lane_back(float v, int k)
{
    static_assert(S == 2 || S == 4, "chains are lane pairs or quads");
    const int i = __float_as_int(v);
    k &= S - 1;
    if (k == 0) return v;
    if (S == 2) return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0xB1, 0xF, 0xF, true));      // [1,0,3,2]
    if (k == 1) return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0x93, 0xF, 0xF, true));      // [3,0,1,2]
    if (k == 2) return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0x4E, 0xF, 0xF, true));      // [2,3,0,1]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, i, 0x39, 0xF, 0xF, true));                  // [1,2,3,0]
}

// The value lane j of the caller's chain holds (j constant after unrolling).
template <int S>
__device__ __forceinline__ float chain_lane_pick(float v, int j)
{
    if (S == 2) return j == 0 ? chain_lane_value<2, 0>(v) : chain_lane_value<2, 1>(v);
    if (j == 0) return chain_lane_value<4, 0>(v);
    if (j == 1) return chain_lane_value<4, 1>(v);
    if (j == 2) return chain_lane_value<4, 2>(v);
    return chain_lane_value<4, 3>(v);
}

// Addressing of the dealt walk.  Per tensor, a wave-uniform 64-bit pointer to the lowest-address row of a tile (so
// that every lane offset is non-negative whatever the direction of the walk) moves by one tile per iteration, and a
// lane's own (group, token, channel) inside a tile is a 32-bit byte offset fixed for the whole walk: a memory
// instruction takes both as they are, and the loop is left with one pointer step per tensor and tile.
template <typename T>
__device__ __forceinline__ T load_at(const T* tile_row, unsigned lane_bytes)
{
    return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(tile_row) + lane_bytes);
}
template <typename T>
__device__ __forceinline__ void store_at(T* tile_row, unsigned lane_bytes, T v)
{
    *reinterpret_cast<T*>(reinterpret_cast<char*>(tile_row) + lane_bytes) = v;
}
// A lane offset has to be a 32-bit value of the block that uses it: widened to 64 bits outside the loop (where the
// compiler would move the widening) it is no longer recognised as the offset operand of a scalar-base access and
// costs a 64-bit vector add per access.  Passing it through an empty asm once per tile keeps it where it is.
__device__ __forceinline__ void keep_narrow(unsigned& lane_bytes) { asm volatile("" : "+v"(lane_bytes)); }

// Tokens per dealt tile, and the shapes that deal their tokens: up to 16 states split over two or four lanes (with more
// states per lane the state updates dominate and the plain walk's smaller register footprint wins).
template <int N, int S>
constexpr int kDealtTile = 8;
template <int N, int S>
constexpr bool kDealtTokens = S > 1 && N <= 16;

typedef float Float4 __attribute__((ext_vector_type(4)));  // a native vector: copies of structs that hold it stay in registers
template <typename IO, int G, int NSTAGE>
struct DealtTile {
    typename IO::T x[G], z[G], dt[G];
    float part[G];
    Float4 bc[NSTAGE];   // the lane's share of the tile's B|C rows on their way to LDS
};

// Whole tiles of tokens [0, count) of the chain's walk, dealt as described above; returns the number of tokens done
// (a multiple of the dealt tile).  On entry and on return c.xh holds the raw x of the three tokens before the current
// position, alike in all lanes of the chain, so the per-token path can take over the remainder.  lds: this wave's
// private 2 * DT * 2N floats.  Two tile register sets are used in turn (the loop body is the pair), so a tile is
// computed from the registers its loads arrived in.
template <int N, int S, int AKIND, typename IO, int MODE>
__device__ __forceinline__ int run_tiles_dealt(const SweepArgs& a, Chain<N, S, AKIND, IO>& c, int count, bool softplus_dt,
                                               float* lds, int lane)
{
    static_assert((S == 2 || S == 4) && MODE != kModeNoOutput, "dealt tiles: lane pairs or quads, output modes");
    using T = typename IO::T;
    constexpr int DT = kDealtTile<N, S>;
    constexpr int NS = N / S, G = DT / S, D = (3 + S - 1) / S;
    constexpr int kRowF4 = 2 * N / 4;
    constexpr int kStage = (DT * kRowF4 + 63) / 64;
    constexpr bool kGated = MODE != kModePartialRaw;
    using Tile = DealtTile<IO, G, kStage>;
    const int total = count / DT * DT;
    if (total == 0) return 0;
    const int sub = (int)c.sub;

    // tap weight or zero per (k tokens back, d groups back)
    float wk[3][D + 1];
#pragma unroll
    for (int k = 1; k <= 3; k++)
#pragma unroll
        for (int d = 0; d <= D; d++) {
            float v = 0.0f;
#pragma unroll
            for (int j = 0; j < S; j++)
                if (dealt_groups_back<S>(j, k) == d) v = sub == j ? c.w4[3 - k] : v;
            wk[k - 1][d] = v;
        }
    // own raw x of the last groups: hist[d] is d groups back once a group's value has been shifted in.  Before the
    // first group, hist[d - 1] is seeded with "group -d": the token before the walk by m + 1 sits in lane
    // (-1 - m) mod S of group -ceil((m + 1) / S).
    float hist[D + 1];
#pragma unroll
    for (int d = 1; d <= D + 1; d++) {
        float v = 0.0f;
#pragma unroll
        for (int j = 0; j < S; j++) {
            const int m = d * S - j - 1;
            if (m >= 0 && m <= 2) v = sub == j ? c.xh[m] : v;
        }
        hist[d - 1] = v;
    }
    // The lane's own token of group q inside a tile's rows, per tensor: bytes above the tile's lowest-address row,
    // plus the lane's channel.  Token q * S + sub of the tile lies that many rows up when the walk ascends in memory,
    // DT - 1 - that many when it descends.
    auto absll = [](long long v) { return v < 0 ? -v : v; };
    auto rows_up = [&](long long step, int token) { return step < 0 ? DT - 1 - token : token; };
    unsigned vx[G], vd[G], vz[G], vo[G], vp[G];
#pragma unroll
    for (int q = 0; q < G; q++) {
        const int t = q * S + sub;
        vx[q] = c.ch_io + (unsigned)rows_up(c.xs, t) * (unsigned)(absll(c.xs) * (long long)sizeof(T));
        vd[q] = c.head_io + (unsigned)rows_up(c.dts, t) * (unsigned)(absll(c.dts) * (long long)sizeof(T));
        vz[q] = c.ch_io + (unsigned)rows_up(c.zs, t) * (unsigned)(absll(c.zs) * (long long)sizeof(T));
        vo[q] = c.ch_io + (unsigned)rows_up(c.os, t) * (unsigned)(absll(c.os) * (long long)sizeof(T));
        vp[q] = c.ch_f32 + (unsigned)rows_up(c.ps, t) * (unsigned)(absll(c.ps) * 4LL);
    }
    // lane q moves float4 number (j*64 + q) of a tile's B|C rows: token (scan order) idx / kRowF4, column idx % kRowF4
    unsigned vbc[kStage];
#pragma unroll
    for (int j = 0; j < kStage; j++) {
        const int idx = min(j * 64 + lane, DT * kRowF4 - 1);
        vbc[j] = (unsigned)rows_up(c.bcs, idx / kRowF4) * (unsigned)(absll(c.bcs) * 4LL) + (unsigned)(idx % kRowF4) * 16u;
    }
    auto lowest = [&](auto* row, long long step) { return step < 0 ? row + (DT - 1) * step : row; };
    // tile pointers: the inputs' run one tile ahead of the outputs' once the first tile has been requested
    const T* xin = lowest(c.xrow, c.xs);
    const T* din = lowest(c.dtrow, c.dts);
    const T* zin = lowest(c.zrow, c.zs);
    const float* pin = lowest(c.prow, c.ps);
    const float* bcin = lowest(c.bcrow, c.bcs);
    T* oout = lowest(c.orow, c.os);
    float* pout = lowest(c.prow, c.ps);
    auto load = [&](Tile& r) {
#pragma unroll
        for (int q = 0; q < G; q++) {
            r.x[q] = load_at(xin, vx[q]);
            r.dt[q] = load_at(din, vd[q]);
            if (mode_reads_z(MODE)) r.z[q] = load_at(zin, vz[q]);
            if (mode_reads_partial(MODE)) r.part[q] = load_at(pin, vp[q]);
        }
#pragma unroll
        for (int j = 0; j < kStage; j++)
            if (DT * kRowF4 % 64 == 0 || j * 64 + lane < DT * kRowF4)
                r.bc[j] = load_at(reinterpret_cast<const Float4*>(bcin), vbc[j]);
        xin += DT * c.xs;
        din += DT * c.dts;
        if (mode_reads_z(MODE)) zin += DT * c.zs;
        if (mode_reads_partial(MODE)) pin += DT * c.ps;
        bcin += DT * c.bcs;
    };
    auto stage_store = [&](int which, const Tile& r) {
#pragma unroll
        for (int j = 0; j < kStage; j++) {
            const int idx = j * 64 + lane;
            if (DT * kRowF4 % 64 == 0 || idx < DT * kRowF4)
                *reinterpret_cast<Float4*>(lds + which * (DT * 2 * N) + idx * 4) = r.bc[j];
        }
        __builtin_amdgcn_wave_barrier();  // other lanes of this wave read these rows next; LDS keeps wave order
    };

    BcRow<NS> row;
    int buf = 0, done = 0;
    // One tile: request the next one into `fill`, compute `cur`, move on.  Returns false after the last tile.
    auto one_tile = [&](const Tile& cur, Tile& fill) -> bool {
        const bool more = done + 2 * DT <= total;
#pragma unroll
        for (int q = 0; q < G; q++) {
            keep_narrow(vx[q]);
            keep_narrow(vd[q]);
            keep_narrow(vz[q]);
            keep_narrow(vo[q]);
            keep_narrow(vp[q]);
        }
#pragma unroll
        for (int j = 0; j < kStage; j++) keep_narrow(vbc[j]);
        if (more) {
            if ((done & (4 * DT - 1)) == 0) take_turn(a);
            load(fill);
        }
        const float* tile_bc = lds + buf * (DT * 2 * N);
        float delta[G];
#pragma unroll
        for (int q = 0; q < G; q++) delta[q] = IO::cvt(cur.dt[q]);
        if (softplus_dt) {
#pragma unroll
            for (int q = 0; q < G; q++) delta[q] = softplus(delta[q] + c.dtb);
        }
#pragma unroll
        for (int q = 0; q < G; q++) {
            // the owner's share of its token: conv window, SiLUs, input and decay factors
#pragma unroll
            for (int d = D; d >= 1; d--) hist[d] = hist[d - 1];
            hist[0] = IO::cvt(cur.x[q]);
            float pre = fmaf(c.w4[3], hist[0], c.cb);
#pragma unroll
            for (int k = 1; k <= 3; k++)
#pragma unroll
                for (int d = 0; d <= D; d++)
                    if (dealt_term_exists<S>(k, d)) pre = fmaf(chain_lane_back<S>(hist[d], k), wk[k - 1][d], pre);
            const float xc = silu(pre);
            const float u = delta[q] * xc;
            float zg = 0.0f, fac = 0.0f;
            if (kGated) zg = silu(IO::cvt(cur.z[q]));
            if (AKIND == kAProgression) fac = fast_exp2(delta[q] * c.d2);        // ratio between neighbouring states
            else if (AKIND == kAScalar) fac = fast_exp2(delta[q] * c.a2[0]);     // the head's decay
            float ys[S];
#pragma unroll
            for (int jt = 0; jt < S; jt++) {
                const int i = q * S + jt;
                BcRow<NS> row_next;
                if (i + 1 < DT) load_bc_lds<N, S>(tile_bc, i + 1, c.sub, row_next);
                const float ui = chain_lane_pick<S>(u, jt);
                float y = 0.0f;
                if (AKIND == kAPerState) {
                    const float di = chain_lane_pick<S>(delta[q], jt);
#pragma unroll
                    for (int n = 0; n < NS; n++) {
                        c.h[n] = fmaf(fast_exp2(di * c.a2[n]), c.h[n], ui * row.v[n]);
                        y = fmaf(row.v[NS + n], c.h[n], y);
                    }
                } else if (AKIND == kAProgression) {
                    const float di = chain_lane_pick<S>(delta[q], jt), ratio = chain_lane_pick<S>(fac, jt);
                    float an = fast_exp2(di * c.a2[0]);
#pragma unroll
                    for (int n = 0; n < NS; n++) {
                        c.h[n] = fmaf(an, c.h[n], ui * row.v[n]);
                        y = fmaf(row.v[NS + n], c.h[n], y);
                        if (n + 1 < NS) an *= ratio;
                    }
                } else {
                    const float an = chain_lane_pick<S>(fac, jt);
#pragma unroll
                    for (int n = 0; n < NS; n++) {
                        c.h[n] = fmaf(an, c.h[n], ui * row.v[n]);
                        y = fmaf(row.v[NS + n], c.h[n], y);
                    }
                }
                ys[jt] = sum_over_chain_lanes<S>(y);
                if (i + 1 < DT) row = row_next;
            }
            // the owner finishes its token
            float y = ys[0];
#pragma unroll
            for (int jt = 1; jt < S; jt++) y = sub == jt ? ys[jt] : y;
            y = fmaf(c.dval, xc, y);
            if (MODE == kModePartialRaw) {
                store_at(pout, vp[q], y);
            } else if (MODE == kModeFinalAddRaw) {
                store_at(oout, vo[q], io_value<IO>((y + cur.part[q]) * zg));
            } else {
                const float g = y * zg;
                if (MODE == kModePartial) store_at(pout, vp[q], g);
                else store_at(oout, vo[q], io_value<IO>(MODE == kModeFinalAdd ? g + cur.part[q] : g));
            }
        }
        done += DT;
        if (MODE == kModePartialRaw || MODE == kModePartial) pout += DT * c.ps;
        else oout += DT * c.os;
        if (!more) return false;
        buf ^= 1;
        stage_store(buf, fill);
        load_bc_lds<N, S>(lds + buf * (DT * 2 * N), 0, c.sub, row);
        return true;
    };

    Tile ta, tb;
    load(ta);
    stage_store(0, ta);
    load_bc_lds<N, S>(lds, 0, c.sub, row);
    while (true) {
        if (!one_tile(ta, tb)) break;
        if (!one_tile(tb, ta)) break;
    }
    // hand the conv history back in the per-token form: the token m + 1 back sits in lane (S - 1 - m) mod S, m / S groups back
#pragma unroll
    for (int m = 0; m < 3; m++) c.xh[m] = chain_lane_pick<S>(hist[m / S], (S - 1 - m % S));
    advance_rows(c, done);
    c.bcrow += done * c.bcs;
    c.tok += done * c.tstep;
    return done;
}

// Tokens of the larger of the two kinds of tile a wave stages B|C rows for (its LDS area holds two of them).
template <int N, int S, int TILE>
constexpr int kStagedTile = kDealtTokens<N, S> && kDealtTile<N, S> > TILE ? kDealtTile<N, S> : TILE;

template <int N, int S, int AKIND, typename IO, int MODE, int TILE, int BCSRC = kBcPrepared>
__device__ __forceinline__ void run_range(const SweepArgs& a, Chain<N, S, AKIND, IO>& c, int count, bool softplus_dt, float* lds,
                                          int lane)
{
    static_assert(BCSRC == kBcPrepared || (S == 1 && N <= 16), "staged rows exist for one lane per chain, <= 16 states");
    constexpr int NS = N / S;
    constexpr int kRowF4 = 2 * N / 4;              // float4s per B|C row
    constexpr int kStage = (TILE * kRowF4 + 63) / 64;  // float4s each lane moves per staged tile
    // With the shallow tile (many waves per SIMD) token_step refills the one scalar row itself; with the deep tile
    // (two or three waves per SIMD, less cover for a scalar load) the next token's row is requested a whole token
    // ahead into a second set of registers.
    constexpr bool kRefill = kBcScalarAhead<N, S> && BCSRC == kBcPrepared && TILE == 4;
    using Tile = RawTile<IO, TILE>;
    if (count <= 0) return;
    int done = 0;
    if constexpr (kDealtTokens<N, S> && MODE != kModeNoOutput && BCSRC == kBcPrepared) {
        done = run_tiles_dealt<N, S, AKIND, IO, MODE>(a, c, count, softplus_dt, lds, lane);
    } else if (count >= TILE) {
        Tile nxt;
        load_tile<N, S, AKIND, IO, MODE, TILE>(c, 0, nxt);
        BcRow<NS> row;
        float4 stage[kStage];
        int buf = 0;
        // lane q moves float4 number (j*64 + q) of the tile: token (scan order) idx / kRowF4, column idx % kRowF4
        auto stage_load = [&](long long ahead) {
#pragma unroll
            for (int j = 0; j < kStage; j++) {
                const int idx = j * 64 + lane;
                if (TILE * kRowF4 % 64 == 0 || idx < TILE * kRowF4)
                    stage[j] = *reinterpret_cast<const float4*>(c.bcrow + (ahead + idx / kRowF4) * c.bcs + (idx % kRowF4) * 4);
            }
        };
        auto stage_store = [&](int which) {
#pragma unroll
            for (int j = 0; j < kStage; j++) {
                const int idx = j * 64 + lane;
                if (TILE * kRowF4 % 64 == 0 || idx < TILE * kRowF4)
                    *reinterpret_cast<float4*>(lds + which * (TILE * 2 * N) + idx * 4) = stage[j];
            }
            __builtin_amdgcn_wave_barrier();  // other lanes of this wave read these rows next; LDS keeps wave order
        };
        if constexpr (S > 1) {
            stage_load(0);
            stage_store(0);
            load_bc_lds<N, S>(lds, 0, c.sub, row);
        } else if constexpr (BCSRC == kBcStaged) {
            load_bc_lds<N, 1>(lds, c.tok, 0, row);
        } else if constexpr (kBcScalarAhead<N, S>) {
            load_bc_scalar<N>(c.bcrow, row);
        }
        while (true) {
            // the tile requested one iteration (or, the first time, a moment) ago; its registers are free for the next
            // request from here on
            const Tile cur = nxt;
            const bool more = done + 2 * TILE <= count;
            if (more) {
                // every fourth tile (the clock read is not free), here because this block starts at a branch anyway
                if ((done & (4 * TILE - 1)) == 0) take_turn(a);
                load_tile<N, S, AKIND, IO, MODE, TILE>(c, TILE, nxt);
                if constexpr (S > 1) stage_load(TILE);
            }
            const float* tile_bc = lds + buf * (TILE * 2 * N);
            const TileRows<TILE> to = tile_rows<TILE>(c.orow, c.os), tpk = tile_rows<TILE>(c.prow, c.ps);
            // Delta of the whole tile up front: one uniform branch per tile instead of one per token
            float delta[TILE];
#pragma unroll
            for (int i = 0; i < TILE; i++) delta[i] = IO::cvt(cur.dt[i]);
            if (softplus_dt) {
                if constexpr (S > 1 && TILE % S == 0) {
                    // the S lanes of a chain need the same TILE values: each evaluates TILE / S of them and hands
                    // them round with quad-permute moves
                    constexpr int kPer = TILE / S;
                    float mine[kPer];
#pragma unroll
                    for (int i = 0; i < kPer; i++) {
                        float v = delta[i];
#pragma unroll
                        for (int j = 1; j < S; j++) v = c.sub == (unsigned)j ? delta[j * kPer + i] : v;
                        mine[i] = softplus(v + c.dtb);
                    }
#pragma unroll
                    for (int i = 0; i < kPer; i++) {
                        delta[i] = chain_lane_value<S, 0>(mine[i]);
                        delta[kPer + i] = chain_lane_value<S, 1>(mine[i]);
                        if constexpr (S == 4) {
                            delta[2 * kPer + i] = chain_lane_value<S, 2>(mine[i]);
                            delta[3 * kPer + i] = chain_lane_value<S, 3>(mine[i]);
                        }
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < TILE; i++) delta[i] = softplus(delta[i] + c.dtb);
                }
            }
#pragma unroll
            for (int i = 0; i < TILE; i++) {
                BcRow<NS> row_next;
                if constexpr (S > 1) {
                    if (i + 1 < TILE) load_bc_lds<N, S>(tile_bc, i + 1, c.sub, row_next);
                } else if constexpr (BCSRC == kBcStaged) {
                    load_bc_lds<N, 1>(lds, done + i + 1 < count ? c.tok + c.tstep : c.tok, 0, row_next);
                }
                // never read past the walk's last token: the row after it may lie outside the buffer
                const float* next = kBcScalarAhead<N, S> ? (done + i + 1 < count ? c.bcrow + c.bcs : c.bcrow) : nullptr;
                if constexpr (kBcScalarAhead<N, S> && BCSRC == kBcPrepared && !kRefill) {
                    load_bc_scalar<N>(next, row_next);
                    __builtin_amdgcn_sched_barrier(0);
                }
                token_step<N, S, AKIND, IO, MODE, kRefill>(c, cur.x[i], delta[i], cur.z[i], cur.part[i], row, next,
                                                  TileSink<IO, TILE>{to, tpk, c.ch_io, c.ch_f32, i});
                if constexpr (S > 1) {
                    if (i + 1 < TILE) row = row_next;
                } else if constexpr (BCSRC == kBcStaged) {
                    row = row_next;
                } else if constexpr (kBcScalarAhead<N, S> && !kRefill) {
                    __builtin_amdgcn_sched_barrier(0);
                    row = row_next;
                }
            }
            done += TILE;
            advance_rows(c, TILE);
            if (!more) break;
            if constexpr (S > 1) {
                buf ^= 1;
                stage_store(buf);
                load_bc_lds<N, S>(lds + buf * (TILE * 2 * N), 0, c.sub, row);
            }
        }
    }
    for (; done < count; done++) {
        typename IO::T xr = *lane_elem(c.xrow, c.ch_io), dr = *lane_elem(c.dtrow, c.head_io), zr = 0;
        float part = 0.0f;
        if (mode_reads_z(MODE)) zr = *lane_elem(c.zrow, c.ch_io);
        if (mode_reads_partial(MODE)) part = *lane_elem(c.prow, c.ch_f32);
        BcRow<NS> row;
        if constexpr (S > 1) load_bc_direct<N, S>(c.bcrow, c.sub, row);
        else if constexpr (BCSRC == kBcStaged) load_bc_lds<N, 1>(lds, c.tok, 0, row);
        else if constexpr (kBcScalarAhead<N, S>) load_bc_scalar<N>(c.bcrow, row);
        float delta = IO::cvt(dr);
        if (softplus_dt) delta = softplus(delta + c.dtb);
        token_step<N, S, AKIND, IO, MODE, false>(c, xr, delta, zr, part, row, nullptr,
                                                 RowSink<IO>{c.orow, c.prow, c.ch_io, c.ch_f32});
        advance_rows(c, 1);
    }
}

// Segment summary without the recurrence (one lane per chain, scalar-register rows).  From a zero start the end state
// of a segment is  S[n] = sum_t exp(A[n] * W_t) * Delta_t xc_t B_t[n],  W_t = the Delta of the tokens that follow t
// in scan order.  Walking the segment from its scan-last token towards its scan-first one, W_t is a running sum and a
// token costs two VALU per state (coefficient step, accumulate) where the recurrence costs three (decay step, input
// product, update).  The conv of a token needs the raw x of the three tokens that precede it in scan order, which
// this walk meets later: a token is folded in three steps after its own x arrived, once the window is complete, with
// its Delta taken from a three-deep delay line.  On entry c is positioned at the segment's scan-first token with
// scan-order steps and a zero state; c.xh holds the raw x of the three tokens before the segment.  On return c.h is
// the end state and c.sum_dt the segment's total Delta.
template <int N, int AKIND, typename IO, int TILE>
__device__ __forceinline__ void summarise_from_the_end(Chain<N, 1, AKIND, IO>& c, int len, bool softplus_dt)
{
    using Tile = RawTile<IO, TILE>;
    // reposition at the scan-last token and walk against the scan order
    c.xrow += (long long)(len - 1) * c.xs;
    c.dtrow += (long long)(len - 1) * c.dts;
    c.bcrow += (long long)(len - 1) * c.bcs;
    c.xs = -c.xs;
    c.dts = -c.dts;
    c.bcs = -c.bcs;
    float xw0 = 0.0f, xw1 = 0.0f, xw2 = 0.0f, xw3 = 0.0f;   // raw x, xw0 the newest (three tokens before the one folded)
    float d1 = 0.0f, d2 = 0.0f, d3 = 0.0f;                   // Delta, d3 the oldest (the token folded next)
    float wsum = 0.0f;                                       // W of the token folded next
    int folded = 0;                                          // tokens folded so far; the next one is scan index len-1-folded
    float brow[N];
    uniform_ro_ptr q = (uniform_ro_ptr)c.bcrow;
#pragma unroll
    for (int n = 0; n < N; n++) brow[n] = q[n];
    auto push = [&](float x, float delta) {
        xw3 = xw2; xw2 = xw1; xw1 = xw0; xw0 = x;
        d3 = d2; d2 = d1; d1 = delta;
    };
    // folds the token whose x sits in xw3 and whose Delta was in d3 before the push that completed its window
    auto fold = [&](float delta) {
        float pre = c.cb;
        pre = fmaf(c.w4[0], xw0, pre);
        pre = fmaf(c.w4[1], xw1, pre);
        pre = fmaf(c.w4[2], xw2, pre);
        pre = fmaf(c.w4[3], xw3, pre);
        const float u = delta * silu(pre);
        if (AKIND == kAPerState) {
#pragma unroll
            for (int n = 0; n < N; n++) c.h[n] = fmaf(fast_exp2(wsum * c.a2[n]) * u, brow[n], c.h[n]);
        } else if (AKIND == kAProgression) {
            float cn = fast_exp2(wsum * c.a2[0]) * u;
            const float ratio = fast_exp2(wsum * c.d2);
#pragma unroll
            for (int n = 0; n < N; n++) {
                c.h[n] = fmaf(cn, brow[n], c.h[n]);
                cn *= ratio;
            }
        } else {
            const float cn = fast_exp2(wsum * c.a2[0]) * u;
#pragma unroll
            for (int n = 0; n < N; n++) c.h[n] = fmaf(cn, brow[n], c.h[n]);
        }
        wsum += delta;
        folded++;
        // the row of the token folded next, into the registers just read (never past the segment's first row)
        __builtin_amdgcn_sched_barrier(0);
        if (folded < len) c.bcrow += c.bcs;
        uniform_ro_ptr nq = (uniform_ro_ptr)c.bcrow;
#pragma unroll
        for (int n = 0; n < N; n++) brow[n] = nq[n];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto delta_of = [&](typename IO::T raw) {
        const float v = IO::cvt(raw);
        return softplus_dt ? softplus(v + c.dtb) : v;
    };
    // the first three tokens only fill the window
    const int lead = min(3, len);
    for (int k = 0; k < lead; k++) {
        push(IO::cvt(*lane_elem(c.xrow, c.ch_io)), delta_of(*lane_elem(c.dtrow, c.head_io)));
        advance_rows(c, 1);
    }
    int left = len - lead;   // tokens whose x is still to come; each arrival completes the window of one token
    if (left >= TILE) {
        Tile nxt;
        load_tile<N, 1, AKIND, IO, kModeNoOutput, TILE>(c, 0, nxt);
        while (true) {
            const Tile cur = nxt;
            const bool more = left >= 2 * TILE;
            if (more) load_tile<N, 1, AKIND, IO, kModeNoOutput, TILE>(c, TILE, nxt);
            float delta[TILE];
#pragma unroll
            for (int i = 0; i < TILE; i++) delta[i] = IO::cvt(cur.dt[i]);
            if (softplus_dt) {
#pragma unroll
                for (int i = 0; i < TILE; i++) delta[i] = softplus(delta[i] + c.dtb);
            }
#pragma unroll
            for (int i = 0; i < TILE; i++) {
                const float due = d3;
                push(IO::cvt(cur.x[i]), delta[i]);
                fold(due);
            }
            left -= TILE;
            advance_rows(c, TILE);
            if (!more) break;
        }
    }
    for (; left > 0; left--) {
        const float due = d3;
        push(IO::cvt(*lane_elem(c.xrow, c.ch_io)), delta_of(*lane_elem(c.dtrow, c.head_io)));
        fold(due);
        advance_rows(c, 1);
    }
    // the tokens before the segment complete the windows of its first three tokens
#pragma unroll
    for (int i = 0; i < 3; i++) {
        const float due = d3;
        push(c.xh[i], 0.0f);
        if (lead + i >= 3 && folded < len) fold(due);   // (segments shorter than three tokens fill the window here)
    }
    c.sum_dt = wsum;
}

// Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  With S lanes per chain
// a wave's row accesses cover only 1/S of a 128-byte line (bf16), so the S channel tiles that share a line are
// given to workgroups 8 apart: same XCD, dispatched together, and the line is fetched from HBM once.  Within each
// group of 8*S workgroups this is a permutation of the tiles; a ragged last group keeps the identity.
template <int S>
__device__ __forceinline__ unsigned xcd_aware_tile(unsigned g, unsigned n)
{
    constexpr unsigned kGroup = 8 * S;
    if (S == 1 || g >= n / kGroup * kGroup) return g;
    return g / kGroup * kGroup + (g % 8) * S + (g / 8) % S;
}

// The channel tile of wave w of this workgroup.  A workgroup holds two adjacent tiles (waves 0 / 1 walk the first
// left-to-right / right-to-left, waves 2 / 3 the second), so each of a CU's four SIMDs gets one wave of every
// workgroup and the SIMDs stay evenly loaded.  With an odd number of tiles the last workgroup's second pair shadows
// the first: same inputs, same values, same addresses.
template <int S>
__device__ __forceinline__ int tile_of_wave(int w, int Dn)
{
    constexpr int kCpw = 64 / S;
    const unsigned pair = xcd_aware_tile<(S + 1) / 2>(blockIdx.x, gridDim.x);
    return min((int)(pair * 2 + (w >> 1)), (Dn + kCpw - 1) / kCpw - 1);
}

// grid (ceil(ceil(Dn / (64/S)) / 2), nseg, batch), block 256.
template <int N, int S, int AKIND, typename IO, int KIND, int TILE, int BCSRC = kBcPrepared>
__device__ __forceinline__ void sweep_body(const SweepArgs& a, float* lds_all, const int w)
{
    const int s = w & 1;
    using T = typename IO::T;
    constexpr int NS = N / S;
    constexpr int kCpw = 64 / S;  // channels per wave
    const int lane = threadIdx.x & 63;
    float* lds = lds_all + (BCSRC == kBcStaged ? w * (kShortCallTokens * 2 * N) : S > 1 ? w * (2 * kStagedTile<N, S, TILE> * 2 * N) : 0);
    const DirArgs& da = a.dir[s];
    const int b = blockIdx.z, seg = blockIdx.y;
    // Lanes past the last channel shadow channel Dn-1: they load the same inputs, compute the same values and
    // store them to the same addresses, so no lane needs masking anywhere below.
    const int tile = tile_of_wave<S>(w, a.Dn);
    const int ch = min((int)(tile * kCpw + lane / S), a.Dn - 1);
    const int sub = lane % S;
    const int head = ch / a.P;
    const int grp = (int)((tile * kCpw) / a.P) / a.HG;  // uniform: a tile never straddles two B/C groups
    const int t0 = seg * a.seg_len;
    const int t1 = min(a.L, t0 + a.seg_len);
    const int len = t1 - t0;
    if (len <= 0) return;
    if (KIND == kSummary) {
        // the end state of the segment a direction scans last feeds no other segment: it is needed only when the
        // forward state is committed
        const bool scanned_last = s == 0 ? seg == a.nseg - 1 : seg == 0;
        if (scanned_last && !(s == 0 && a.h_out)) return;
    }
    const int step = s == 0 ? 1 : -1;
    const int tstart = s == 0 ? t0 : t1 - 1;

    Chain<N, S, AKIND, IO> c;
    c.ch_io = (unsigned)ch * (unsigned)sizeof(T);
    c.head_io = (unsigned)head * (unsigned)sizeof(T);
    c.ch_f32 = (unsigned)ch * 4u;
    c.sub = sub;
    // per-lane constants
    {
        const int K = a.K;
#pragma unroll
        for (int i = 0; i < 4; i++) c.w4[3 - i] = i < K ? da.conv_w[(size_t)ch * K + (K - 1 - i)] : 0.0f;
        c.cb = da.conv_b ? da.conv_b[ch] : 0.0f;
        c.dval = da.D[a.d_per_head ? head : ch];
        c.dtb = (a.dt_softplus && da.dt_bias) ? da.dt_bias[head] : 0.0f;
        c.d2 = 0.0f;
        if (AKIND == kAPerState) {
#pragma unroll
            for (int n = 0; n < NS; n++) c.a2[n] = da.A[(size_t)head * N + sub * NS + n] * kLog2e;
        } else if (AKIND == kAProgression) {
            c.a2[0] = da.A[(size_t)head * N + sub * NS] * kLog2e;
            c.d2 = (da.A[(size_t)head * N + 1] - da.A[(size_t)head * N]) * kLog2e;
        } else {
            c.a2[0] = da.A[head] * kLog2e;
        }
        c.sum_dt = 0.0f;
    }
    // initial state
    {
        const float* src = nullptr;
        if (KIND == kSweep) {
            if (a.nseg > 1) src = a.carry + ((((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch) * N + sub * NS;
            else if (s == 0 && a.h_in) src = a.h_in + ((size_t)b * a.Dn + ch) * N + sub * NS;
        }
#pragma unroll
        for (int n = 0; n < NS; n++) c.h[n] = src ? src[n] : 0.0f;
    }
    // conv history: the K-1 raw tokens that precede the walk's first token in scan order
    {
        // all requested together from clamped (always valid) addresses, then selected: a short call cannot afford to
        // wait for them one after the other
        const T* xb = (const T*)da.x.p + (size_t)b * da.x.sb + ch;
        const bool cached_tail = s == 0 && a.tail_in != nullptr && a.K > 1;
        T from_seq[3], from_tail[3] = {0, 0, 0};
#pragma unroll
        for (int i = 0; i < 3; i++) from_seq[i] = xb[(long long)min(max(tstart - step * (1 + i), 0), a.L - 1) * da.x.st];
        if (cached_tail) {
#pragma unroll
            for (int i = 0; i < 3; i++)
                from_tail[i] = ((const T*)a.tail_in)[((size_t)b * (a.K - 1) + min(max(a.K - 1 + tstart - step * (1 + i), 0), a.K - 2)) *
                                                         a.tail_ch + ch];
        }
#pragma unroll
        for (int i = 0; i < 3; i++) {
            const int t = tstart - step * (1 + i);
            float v = 0.0f;
            if (i < a.K - 1) {
                if (t >= 0 && t < a.L) v = IO::cvt(from_seq[i]);
                else if (t < 0 && cached_tail) v = IO::cvt(from_tail[i]);
            }
            c.xh[i] = v;
        }
    }
    // wave-uniform row pointers at the walk's first token, and signed per-token steps
    c.xs = step * da.x.st;
    c.zs = step * da.z.st;
    c.dts = step * da.dt.st;
    c.os = step * a.out_st;
    c.ps = step * (long long)a.Dn;
    c.bcs = step * (long long)(a.G * 2 * N);
    c.xrow = (const T*)da.x.p + (size_t)b * da.x.sb + (long long)tstart * da.x.st;
    c.zrow = (const T*)da.z.p + (size_t)b * da.z.sb + (long long)tstart * da.z.st;
    c.dtrow = (const T*)da.dt.p + (size_t)b * da.dt.sb + (long long)tstart * da.dt.st;
    c.orow = (T*)a.out + (size_t)b * a.out_sb + (long long)tstart * a.out_st + (a.separate ? s * a.Dn : 0);
    c.prow = a.partial + ((size_t)b * a.L + tstart) * a.Dn;
    c.bcrow = da.bc + (((size_t)b * a.L + tstart) * a.G + grp) * (2 * N);
    c.tok = tstart;
    c.tstep = step;
    if constexpr (BCSRC == kBcStaged) {
        // this wave's own fp32 copy of its direction's B|C rows of the whole (short) call, indexed by token
        const T* bsrc = (const T*)da.Braw.p + (size_t)b * da.Braw.sb + grp * N;
        const T* csrc = (const T*)da.Craw.p + (size_t)b * da.Craw.sb + grp * N;
        // every load is requested before the first value is used: the call is too short to wait for them one by one
        constexpr int kPerLane = kShortCallTokens * 2 * N / 64;
        const int count = a.L * 2 * N;
        T raw[kPerLane];
#pragma unroll
        for (int j = 0; j < kPerLane; j++) {
            if (j * 64 >= count) break;
            const int idx = min(j * 64 + lane, count - 1);
            const int t = idx / (2 * N), col = idx % (2 * N);
            raw[j] = col < N ? bsrc[(long long)t * da.Braw.st + col] : csrc[(long long)t * da.Craw.st + col - N];
        }
#pragma unroll
        for (int j = 0; j < kPerLane; j++) {
            if (j * 64 >= count) break;
            if (j * 64 + lane < count) lds[j * 64 + lane] = IO::cvt(raw[j]);
        }
        __builtin_amdgcn_wave_barrier();  // read back by other lanes of this wave only; LDS keeps wave order
    }
    const bool sp = a.dt_softplus != 0;

    if (KIND == kSummary) {
        if constexpr (kBcScalarAhead<N, S>) summarise_from_the_end<N, AKIND, IO, TILE>(c, len, sp);
        else run_range<N, S, AKIND, IO, kModeNoOutput, TILE>(a, c, len, sp, lds, lane);
        float* dst = a.carry + ((((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch) * N + sub * NS;
#pragma unroll
        for (int n = 0; n < NS; n++) dst[n] = c.h[n];
        a.sumdt[(((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch] = c.sum_dt;
        return;
    }

    if (a.separate) {
        run_range<N, S, AKIND, IO, kModeFinalOnly, TILE, BCSRC>(a, c, len, sp, lds, lane);
    } else {
        // forward parks [t0, m), reverse parks [m, t1); then each finishes the other's half
        const int n_first = s == 0 ? (len + 1) / 2 : len / 2;
        if (a.raw_partial) run_range<N, S, AKIND, IO, kModePartialRaw, TILE, BCSRC>(a, c, n_first, sp, lds, lane);
        else run_range<N, S, AKIND, IO, kModePartial, TILE, BCSRC>(a, c, n_first, sp, lds, lane);
        __syncthreads();  // workgroup-scope release/acquire: the other wave's partials are visible from here on
        if (a.raw_partial) run_range<N, S, AKIND, IO, kModeFinalAddRaw, TILE, BCSRC>(a, c, len - n_first, sp, lds, lane);
        else run_range<N, S, AKIND, IO, kModeFinalAdd, TILE, BCSRC>(a, c, len - n_first, sp, lds, lane);
    }
    if (s == 0 && a.nseg == 1 && a.h_out) {
        float* dst = a.h_out + ((size_t)b * a.Dn + ch) * N + sub * NS;
#pragma unroll
        for (int n = 0; n < NS; n++) dst[n] = c.h[n];
    }
}

// The progression form of the decay is used for bf16 I/O and up to 32 states (its rounding error grows with the state
// index, which bf16 output hides and an fp32 comparison would not).
template <int N, typename IO>
constexpr bool kProgressionEligible = (N >= 2 && N <= 32 && sizeof(typename IO::T) == 2);

// Register budget of the sweep where the tokens are dealt: lane quads are meant to put four waves on a SIMD (128
// registers), lane pairs three (168; measured at d_inner 4096, L 8192 against a budget of two waves: batch 12
// 2.93 -> 2.52 ms, batch 8 1.82 -> 1.77 ms).
template <int N, int S, int KIND>
constexpr int kSweepMinWaves = KIND == kSweep && kDealtTokens<N, S> ? (S == 4 ? 4 : 3) : 1;

template <int N, int S, int AKIND, typename IO, int KIND, int TILE, int BCSRC = kBcPrepared>
__global__ __launch_bounds__(256, (kSweepMinWaves<N, S, KIND>)) void sweep_kernel(const SweepArgs a)
{
    __shared__ __attribute__((aligned(16))) float lds_all[BCSRC == kBcStaged ? 4 * kShortCallTokens * 2 * N
                                                          : S > 1            ? 4 * 2 * kStagedTile<N, S, TILE> * 2 * N
                                                                             : 4];
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if constexpr (AKIND == kAPerState && kProgressionEligible<N, IO>) {
        // Every lane checks its own chain's A row: A[h, n] == fma(n, A[h, 1] - A[h, 0], A[h, 0]) for all n.  The wave takes
        // the two-exponential form only if all of its chains qualify (a wave-uniform vote, no extra launch).
        if (a.try_progression) {
            const int ch = min((int)(tile_of_wave<S>(w, a.Dn) * (64 / S) + (threadIdx.x & 63) / S), a.Dn - 1);
            const float* row = a.dir[w & 1].A + (size_t)(ch / a.P) * N;
            const float first = row[0], step = row[1] - row[0];
            bool ok = true;
#pragma unroll
            for (int n = 0; n < N; n++) ok &= row[n] == fmaf((float)n, step, first);
            if (__all(ok)) {
                sweep_body<N, S, kAProgression, IO, KIND, TILE, BCSRC>(a, lds_all, w);
                return;
            }
        }
    }
    sweep_body<N, S, AKIND, IO, KIND, TILE, BCSRC>(a, lds_all, w);
}

// Stitch time segments: carry[s][b][seg] holds each segment's end state from a zero start (summary pass); replace it
// by the state entering the segment, folding (decay product, end state) pairs in scan order:
//   h_next = exp(A * sum_dt_seg) * h + S_seg.
struct CarryArgs {
    float* carry;
    const float* sumdt;
    const float* A[2];
    const float* h_in;
    float* h_out;
    int batch, nseg, Dn, P;
};

// One thread per (direction, batch, channel, state).  A thread's walk over the segments is a dependent chain, but the
// addresses are not: the summaries of kAhead segments are requested together, then folded in order.
template <int N, int AKIND>
__global__ __launch_bounds__(256) void carry_kernel(const CarryArgs a)
{
    constexpr int kAhead = 16;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = 2LL * a.batch * a.Dn * N;
    if (idx >= total) return;
    const int n = (int)(idx % N);
    const int ch = (int)((idx / N) % a.Dn);
    const int b = (int)((idx / ((long long)N * a.Dn)) % a.batch);
    const int s = (int)(idx / ((long long)N * a.Dn * a.batch));
    const int head = ch / a.P;
    const float a2 = a.A[s][AKIND == 0 ? (size_t)head * N + n : (size_t)head] * kLog2e;
    float h = (s == 0 && a.h_in) ? a.h_in[((size_t)b * a.Dn + ch) * N + n] : 0.0f;
    const size_t first_row = ((size_t)s * a.batch + b) * a.nseg * a.Dn + ch;   // segment seg: first_row + seg * Dn
    auto row_of = [&](int i) { return first_row + (size_t)(s == 0 ? i : a.nseg - 1 - i) * a.Dn; };
    for (int i0 = 0; i0 < a.nseg; i0 += kAhead) {
        float end_state[kAhead], sd[kAhead];
#pragma unroll
        for (int j = 0; j < kAhead; j++) {
            const size_t row = row_of(min(i0 + j, a.nseg - 1));
            end_state[j] = a.carry[row * N + n];
            sd[j] = a.sumdt[row];
        }
#pragma unroll
        for (int j = 0; j < kAhead; j++) {
            if (i0 + j < a.nseg) {
                a.carry[row_of(i0 + j) * N + n] = h;
                h = fmaf(fast_exp2(sd[j] * a2), h, end_state[j]);
            }
        }
    }
    if (s == 0 && a.h_out) a.h_out[((size_t)b * a.Dn + ch) * N + n] = h;
}

// B and C rows as the scan consumes them: fp32, [batch][L][G][B(0..N) | C(0..N)], raw values or conv + SiLU'd like x
// (Mamba-2 form: conv channels d_inner.. are B then C).  One thread per output value.
struct PrepArgs {
    TensorArg B, C;
    const float* conv_w;  // full [conv_ch][K] table of this direction (rows Dn.. used) or null when !conv_bc
    const float* conv_b;
    const void* tail_in;  // causal direction of the block variant, or null
    float* dst;
    int batch, L, G, N, K, Dn, tail_ch, conv_bc, dir;  // dir +1 / -1
};

template <typename IO>
__global__ __launch_bounds__(256) void prep_bc_kernel(const PrepArgs a)
{
    using T = typename IO::T;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int GN = a.G * a.N;
    const long long total = (long long)a.batch * a.L * 2 * GN;
    if (idx >= total) return;
    const int n = (int)(idx % a.N);
    const int which = (int)((idx / a.N) % 2);
    const int g = (int)((idx / (2 * a.N)) % a.G);
    const int t = (int)((idx / (2LL * GN)) % a.L);
    const int b = (int)(idx / (2LL * GN * a.L));
    const TensorArg& src = which ? a.C : a.B;
    const int j = g * a.N + n;
    const T* base = (const T*)src.p + (size_t)b * src.sb + j;
    float v;
    if (!a.conv_bc) {
        v = IO::ld(base + (long long)t * src.st);
    } else {
        const int row = a.Dn + which * GN + j;
        float acc = a.conv_b ? a.conv_b[row] : 0.0f;
        for (int k = 0; k < a.K; k++) {
            const int tt = t - a.dir * (a.K - 1 - k);
            float xv = 0.0f;
            if (tt >= 0 && tt < a.L) xv = IO::ld(base + (long long)tt * src.st);
            else if (tt < 0 && a.dir > 0 && a.tail_in)
                xv = IO::ld((const T*)a.tail_in + ((size_t)b * (a.K - 1) + (a.K - 1 + tt)) * a.tail_ch + row);
            acc = fmaf(a.conv_w[(size_t)row * a.K + k], xv, acc);
        }
        v = silu(acc);
    }
    a.dst[idx] = v;
}

// tail_out = last K-1 raw tokens of (tail_in || block); one thread per (batch, tail channel), reads before writes so
// tail_out may alias tail_in.
struct TailArgs {
    TensorArg x, B, C;
    const void* tail_in;
    void* tail_out;
    int batch, L, K, Dn, GN, tail_ch;
};

template <typename IO>
__global__ __launch_bounds__(256) void tail_kernel(const TailArgs a)
{
    using T = typename IO::T;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)a.batch * a.tail_ch) return;
    const int c = (int)(idx % a.tail_ch);
    const int b = (int)(idx / a.tail_ch);
    const T* src;
    long long st;
    if (c < a.Dn) { src = (const T*)a.x.p + (size_t)b * a.x.sb + c; st = a.x.st; }
    else if (c < a.Dn + a.GN) { src = (const T*)a.B.p + (size_t)b * a.B.sb + (c - a.Dn); st = a.B.st; }
    else { src = (const T*)a.C.p + (size_t)b * a.C.sb + (c - a.Dn - a.GN); st = a.C.st; }
    T keep[3];
#pragma unroll
    for (int q = 0; q < 3; q++) {
        T v = 0;
        if (q < a.K - 1) {
            const int pos = a.L + q;  // position in the stream tail_in (K-1 tokens) || block (L tokens)
            if (pos >= a.K - 1) v = src[(long long)(pos - (a.K - 1)) * st];
            else if (a.tail_in) v = ((const T*)a.tail_in)[((size_t)b * (a.K - 1) + pos) * a.tail_ch + c];
        }
        keep[q] = v;
    }
#pragma unroll
    for (int q = 0; q < 3; q++)
        if (q < a.K - 1) ((T*)a.tail_out)[((size_t)b * (a.K - 1) + q) * a.tail_ch + c] = keep[q];
}

}  // namespace bm
