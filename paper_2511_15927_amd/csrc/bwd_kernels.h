// Gradients of the bidirectional mixer path in the selective-scan layout (one head per channel: Delta, A and D per
// channel; B and C shared by the channels of a group; no conv on B and C), for gfx950.
//
// The paper trains these models (App. A.2) but gives no backward algorithm; what is computed here is the chain rule of
// the forward definition (Sec. 3.2 eqs. 4-6 in the concrete selective form), evaluated in the reverse of each
// direction's scan order.  With t+ the token after t in scan order, t- the one before, and dg_t the gradient of the
// gated output of the direction:
//   dz_t = dg_t y_t silu'(z_t)                       dy_t = dg_t silu(z_t)
//   dh_t[n] = C_t[n] dy_t + a_{t+}[n] dh_{t+}[n]
//   dC_t[n] += sum_channels dy_t h_t[n]              dB_t[n] += sum_channels dh_t[n] Delta_t xc_t
//   dA[n] += dh_t[n] h_{t-}[n] a_t[n] Delta_t        dD += dy_t xc_t
//   dDelta_t = sum_n dh_t[n] (h_{t-}[n] a_t[n] A[n] + B_t[n] xc_t)
//   dxc_t = D dy_t + sum_n dh_t[n] Delta_t B_t[n]    dpre_t = dxc_t silu'(pre_t)
//   dx_t = sum_j w[K-1-j] dpre_{t + j steps}         dw[k] += dpre_t x_{t - (K-1-k) steps},  dcb += dpre_t
//
// Mapping: a lane is one (direction, batch, channel) chain, as in the forward sweep with one lane per chain (two
// lanes per chain in the state pass for 8 and 16 states).  The backward recurrence needs the states in the reverse of
// the order the forward recurrence makes them, so
//   bwd_state_kernel  walks each chain forward and stores the state entering every chunk of kBwdChunk tokens;
//   bwd_kernel        takes the chunks last to first: it recomputes a chunk's states from the stored one into
//                     registers (kBwdChunk * N values per lane) and then walks the chunk backwards.
// dB_t and dC_t are sums over the channels of a group: each wave adds its 64 channels with a reduce-scatter over its
// lanes and stores the sums into its own slot of a partial buffer; bwd_bc_kernel adds the slots in a fixed order (no
// atomics on activation gradients: the result does not depend on timing).  Parameter gradients are kept per lane and
// added atomically once per chain (the sum over the batch).  When both directions read the same activations their
// gradients of x, z and Delta have to be added: the two waves of a channel tile walk the tokens in opposite orders
// and meet in the middle, as in the forward sweep; each parks its fp32 values for the half it reaches first and, past
// one workgroup barrier, adds what the other parked to its own values for the other half and rounds once to the I/O dtype.
#pragma once
#include "kernels.h"

namespace bm {

// The fp32 gradients of x, z and Delta of one (token, channel) as one direction leaves them for the other to add.
struct Parked {
    float dx, dz, ddt;
};

struct BwdArgs {
    DirArgs dir[2];          // x, z, dt views, prepared fp32 B|C rows and parameters of each direction
    TensorArg dout;          // [batch][L][Dn] (ADD) or [batch][L][2 Dn] (SEPARATE), I/O dtype
    float* state;            // [2][batch][nchunk][Dn][N]: the state entering each chunk (scan order)
    Parked* parked;          // [batch][L][Dn]: values of the direction that reaches a token first (park only)
    TensorArg gdx[2], gdz[2], gddt[2];   // the caller's gradient views per direction (equal when park)
    int park;                // both directions read the same activations: their gradients are added (see above)
    float* bc_part[2];       // per direction: [batch][L][G][slots][2N] fp32 partial sums of dB | dC, one slot per wave
    int bc_slots;            // slots per group: channel tiles of a group (x 2 when both directions feed one buffer)
    int bc_slot_of_rev;      // slot offset of the reverse direction's waves (0 when it has a buffer of its own)
    float* dA[2];            // [Dn][N]
    float* dD[2];            // [Dn]
    float* dconv_w[2];       // [Dn][K]
    float* dconv_b[2];       // [Dn] or null
    float* ddt_bias[2];      // [Dn] or null
    int L, Dn, G, K, nchunk, dt_softplus, separate;
};

// Tokens per chunk: (chunk + 1) * N state values per lane live in registers during the walk.  DENSE is the form for
// launches with more waves than SIMDs: it has to leave room for a second wave on the SIMD (256 registers), which for 16
// states means chunks of four tokens and twice the stored states (and eight instead of sixteen for 4).  Measured at d_inner 4096 and 64 K tokens: batch 8
// (one wave per SIMD) 17.2 ms in the plain form, 18.8 ms in the dense one; batch 16 and 32: 17.2 against 13.7 ms.
template <int N, bool DENSE>
constexpr int kBwdChunk = DENSE ? (N <= 8 ? 8 : 4) : (N <= 4 ? 16 : 8);

__device__ __forceinline__ float dsilu(float v)
{
    const float s = __builtin_amdgcn_rcpf(1.0f + fast_exp2(-kLog2e * v));
    return s * fmaf(v, 1.0f - s, 1.0f);
}
__device__ __forceinline__ float sigmoidf(float v) { return __builtin_amdgcn_rcpf(1.0f + fast_exp2(-kLog2e * v)); }

// Sums NV values per lane over the 64 lanes of the wave and leaves the total of value j in the lanes
// j * (64 / NV) ... (j + 1) * (64 / NV) - 1 (returned by every lane: the total of value lane / (64 / NV)).
// A reduce-scatter: each step halves the values a lane still carries.  The lane whose bit is clear keeps the first half
// and receives its partner's first half, the other lane the second half, so NV - 1 + log2(64 / NV) adds do the work of
// 6 * NV.  Partners: the other 32-lane half and the other row of 16 by the swap instructions of gfx950, then inside a
// row by lane-permute operands (selection by lane group through their bank mask where the bit picks banks).
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ float lane_permuted(float old, float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(x), CTRL, ROW_MASK, BANK_MASK, false));
}
template <int CTRL>
__device__ __forceinline__ float from_partner(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
template <int NV>
__device__ __forceinline__ float wave_reduce_scatter(float (&v)[NV], int lane)
{
    static_assert(NV == 8 || NV == 16 || NV == 32, "8, 16 or 32 values per lane");
    // lane bit 5: the other half of the wave
#pragma unroll
    for (int i = 0; i < NV / 2; i++) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[i]), __float_as_uint(v[NV / 2 + i]), false, false);
        v[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    // lane bit 4: the neighbouring row of 16
#pragma unroll
    for (int i = 0; i < NV / 4; i++) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[i]), __float_as_uint(v[NV / 4 + i]), false, false);
        v[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    // lane bit 3: banks 2 and 3 of a row keep the second half; the partner is 8 lanes away (row rotate by 8)
#pragma unroll
    for (int i = 0; i < NV / 8; i++) {
        const float keep = lane_permuted<0xE4, 0xF, 0xC>(v[i], v[NV / 8 + i]);
        const float send = lane_permuted<0xE4, 0xF, 0xC>(v[NV / 8 + i], v[i]);
        v[i] = keep + from_partner<0x128>(send);
    }
    if constexpr (NV >= 16) {
        // lane bit 2: banks 1 and 3; the partner is the mirror lane of the other bank of the half row
#pragma unroll
        for (int i = 0; i < NV / 16; i++) {
            const float keep = lane_permuted<0xE4, 0xF, 0xA>(v[i], v[NV / 16 + i]);
            const float send = lane_permuted<0xE4, 0xF, 0xA>(v[NV / 16 + i], v[i]);
            v[i] = keep + from_partner<0x141>(send);
        }
    }
    if constexpr (NV >= 32) {
        // lane bit 1: inside a quad
        const bool upper = (lane & 2) != 0;
        const float keep = upper ? v[1] : v[0], send = upper ? v[0] : v[1];
        v[0] = keep + from_partner<0x4E>(send);
    }
    // what is left of the lane index carries the same value: plain sums, quads first (the mirror needs equal quads)
    float t = v[0];
    t += from_partner<0xB1>(t);                              // quad_perm [1,0,3,2]
    if constexpr (NV <= 16) t += from_partner<0x4E>(t);     // quad_perm [2,3,0,1]
    if constexpr (NV <= 8) t += from_partner<0x141>(t);     // row_half_mirror
    return t;
}

// The per-lane view of one chain shared by both kernels: constants, the scan-order token walk and the forward step.
template <int N, typename IO>
struct BwdChain {
    using T = typename IO::T;
    float a2[N];                 // A * log2(e)
    float w4[4], cb, dval, dtb;  // conv taps (w4[3] on the current token), conv bias, D, Delta bias
    const T *xb, *zb, *dtb_ptr;  // the lane's element of token 0 of this batch element
    long long xs, zs, dts;       // token strides (elements)
    const float* bc;             // prepared B|C rows of this batch element and group: row t at bc + t * bcs
    long long bcs;
    int L, dir;

    __device__ __forceinline__ int token(int scan_index) const { return dir > 0 ? scan_index : L - 1 - scan_index; }
    __device__ __forceinline__ float raw_x(int scan_index) const
    {
        return (scan_index >= 0 && scan_index < L) ? IO::cvt(xb[(long long)token(scan_index) * xs]) : 0.0f;
    }
    __device__ __forceinline__ float delta_of(float raw, bool softplus_dt) const { return softplus_dt ? softplus(raw + dtb) : raw; }
    __device__ __forceinline__ uniform_ro_ptr row(int scan_index) const
    {
        return (uniform_ro_ptr)(bc + (long long)token(scan_index) * bcs);
    }
};

// S lanes per chain: a wave's tile is 64 / S channels, lane l on channel l / S of it.
template <int N, typename IO, int S = 1>
__device__ __forceinline__ bool bwd_chain_setup(const BwdArgs& a, int w, BwdChain<N, IO>& c, int& s, int& b, int& ch, bool& valid)
{
    using T = typename IO::T;
    constexpr int CPW = 64 / S;
    s = w & 1;
    b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    int tile = (int)blockIdx.x * 2 + (w >> 1);
    const bool exists = tile * CPW < a.Dn;               // the second tile of the last workgroup may not exist:
    if (!exists) tile -= 1;                              // its waves shadow the first (they compute and store nothing)
    valid = exists && tile * CPW + lane / S < a.Dn;
    ch = min(tile * CPW + lane / S, a.Dn - 1);            // lanes past the last channel shadow it and contribute nothing
    const DirArgs& da = a.dir[s];
    const int grp = (tile * CPW) / (a.Dn / a.G);         // uniform: a tile never straddles two B/C groups
#pragma unroll
    for (int n = 0; n < N; n++) c.a2[n] = da.A[(size_t)ch * N + n] * kLog2e;
#pragma unroll
    for (int i = 0; i < 4; i++) c.w4[3 - i] = i < a.K ? da.conv_w[(size_t)ch * a.K + (a.K - 1 - i)] : 0.0f;
    c.cb = da.conv_b ? da.conv_b[ch] : 0.0f;
    c.dval = da.D[ch];
    c.dtb = (a.dt_softplus && da.dt_bias) ? da.dt_bias[ch] : 0.0f;
    c.xb = (const T*)da.x.p + (size_t)b * da.x.sb + ch;
    c.zb = (const T*)da.z.p + (size_t)b * da.z.sb + ch;
    c.dtb_ptr = (const T*)da.dt.p + (size_t)b * da.dt.sb + ch;
    c.xs = da.x.st; c.zs = da.z.st; c.dts = da.dt.st;
    c.bcs = (long long)a.G * 2 * N;
    c.bc = da.bc + ((size_t)b * a.L * a.G + grp) * (2 * N);
    c.L = a.L;
    c.dir = s == 0 ? 1 : -1;
    return exists;
}

// Lanes per chain of the state pass.  This pass has no sums across channels, so splitting the states of a chain over
// two lanes costs only the repeated per-channel part (conv, SiLU, Delta: a third of the stream) and puts two waves on
// every SIMD where one lane per chain leaves one, which issues an instruction only every seven cycles.
template <int N>
constexpr int kBwdStateLanes = N >= 8 ? 2 : 1;

// grid (ceil(ceil(Dn / (64 / S)) / 2), 1, batch), block 256: waves 0 / 1 the forward / reverse chain of one channel
// tile, waves 2 / 3 those of the next; S = kBwdStateLanes<N>, lane l of a wave holds states (l % S) * N / S ... of its chain.
template <int N, typename IO, bool DENSE>
__global__ __launch_bounds__(256, kBwdStateLanes<N>) void bwd_state_kernel(const BwdArgs a)
{
    constexpr int CT = kBwdChunk<N, DENSE>;
    constexpr int S = kBwdStateLanes<N>;
    constexpr int NS = N / S;
    static_assert(NS % 4 == 0, "a lane's states are loaded and stored four at a time");
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    BwdChain<N, IO> c;
    int s, b, ch;
    bool valid;
    if (!bwd_chain_setup<N, IO, S>(a, w, c, s, b, ch, valid)) return;
    const bool sp = a.dt_softplus != 0;
    const int part = (int)(threadIdx.x & 63) % S;        // which NS of the chain's states this lane holds
    float a2[NS], h[NS];
#pragma unroll
    for (int n = 0; n < NS; n++) {
        a2[n] = c.a2[n];
#pragma unroll
        for (int e = 1; e < S; e++) a2[n] = part == e ? c.a2[e * NS + n] : a2[n];
        h[n] = 0.0f;
    }
    float x1 = 0.0f, x2 = 0.0f, x3 = 0.0f;   // raw x one, two, three tokens back in scan order
    float* dst = a.state + (((size_t)s * gridDim.z + b) * a.nchunk * a.Dn + ch) * N + part * NS;
    // A SIMD with one or two waves has little to hide a memory round trip behind: the activations of the next chunk
    // are requested before the current chunk is worked through.  That includes the chunk's B rows: the same address
    // in every lane of a part, but as scalar loads their round trips would lie open in front of every other token (a
    // wave waits for all of its scalar loads at once, so none can be kept in flight across a use); as vector loads
    // into the registers such a SIMD has to spare they arrive a chunk early.
    typename IO::T xr[CT], dr[CT], xnext[CT], dnext[CT];
    Float4 br[CT][NS / 4], bnext[CT][NS / 4];
    unsigned in_vgpr = (unsigned)(part * NS * sizeof(float));
    keep_narrow(in_vgpr);                                // an offset the compiler cannot prove uniform
    auto request = [&](typename IO::T (&xq)[CT], typename IO::T (&dq)[CT], Float4 (&bq)[CT][NS / 4], int k) {
#pragma unroll
        for (int i = 0; i < CT; i++) {
            const long long t = c.token(min(k * CT + i, a.L - 1));
            xq[i] = c.xb[t * c.xs];
            dq[i] = c.dtb_ptr[t * c.dts];
            const Float4* row = (const Float4*)((const char*)(c.bc + t * c.bcs) + in_vgpr);
#pragma unroll
            for (int q = 0; q < NS / 4; q++) bq[i][q] = row[q];
        }
    };
    request(xr, dr, br, 0);
    for (int k = 0; k < a.nchunk; k++) {
        if (valid) {
#pragma unroll
            for (int n = 0; n < NS; n++) dst[n] = h[n];
        }
        dst += (size_t)a.Dn * N;
        if (k == a.nchunk - 1) break;    // the state after the last chunk feeds nothing
        request(xnext, dnext, bnext, k + 1);
#pragma unroll
        for (int i = 0; i < CT; i++) {
            if (k * CT + i >= a.L) break;
            const float x0 = IO::cvt(xr[i]);
            const float pre = fmaf(c.w4[0], x3, fmaf(c.w4[1], x2, fmaf(c.w4[2], x1, fmaf(c.w4[3], x0, c.cb))));
            x3 = x2; x2 = x1; x1 = x0;
            const float xc = silu(pre);
            const float delta = c.delta_of(IO::cvt(dr[i]), sp);
            const float u = delta * xc;
#pragma unroll
            for (int n = 0; n < NS; n++) h[n] = fmaf(fast_exp2(delta * a2[n]), h[n], u * br[i][n / 4][n % 4]);
        }
#pragma unroll
        for (int i = 0; i < CT; i++) {
            xr[i] = xnext[i];
            dr[i] = dnext[i];
#pragma unroll
            for (int q = 0; q < NS / 4; q++) br[i][q] = bnext[i][q];
        }
    }
}

template <int N, typename IO, bool DENSE>
__global__ __launch_bounds__(256, DENSE ? 2 : 1) void bwd_kernel(const BwdArgs a)
{
    using T = typename IO::T;
    constexpr int CT = kBwdChunk<N, DENSE>;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    BwdChain<N, IO> c;
    int s, b, ch;
    bool valid;
    // a wave without a tile of its own still runs (as a shadow of its neighbour): the barrier below counts four waves
    const bool exists = bwd_chain_setup<N, IO>(a, w, c, s, b, ch, valid);
    const bool sp = a.dt_softplus != 0;
    const int my_tile = min((int)blockIdx.x * 2 + (w >> 1), (a.Dn + 63) / 64 - 1);
    const int grp = my_tile * 64 / (a.Dn / a.G);
    // Addresses: every tensor is walked through a wave-uniform byte pointer (kept in scalar registers and stepped by
    // scalar adds) plus a byte offset of the lane that is fixed for the whole walk.  Per-lane pointers indexed by the
    // token cost a few scalar multiplies per access, a fifth of this kernel's instructions when it was written that
    // way.  (Forcing the stores into the scalar-base form as well, by keeping the lane offsets 32 bits wide in the
    // blocks of the stores, was measured slower: the pointers then stay live in scalar registers up to each store and
    // the B and C rows push them out into lanes of a vector register.)
    const DirArgs& da = a.dir[s];
    unsigned lo_t = (unsigned)(ch * sizeof(T));                              // x, z, dt, dout, dx, dz, ddt
    unsigned lo_pk = (unsigned)(ch * sizeof(Parked));
    unsigned lo_state = (unsigned)(ch * N * sizeof(float));
    constexpr int kLanesPerValue = 64 / (2 * N);
    unsigned lo_part = (unsigned)((lane / kLanesPerValue) * sizeof(float));
    struct Walked {
        const char* base;    // token 0 of this batch element (and direction, where the tensor has one half per direction)
        int stride;          // bytes per token (the host bounds token strides at 2^26 elements, channels included)
    };
    const Walked wx{(const char*)da.x.p + (size_t)b * da.x.sb * sizeof(T), (int)(da.x.st * (long long)sizeof(T))};
    const Walked wdt{(const char*)da.dt.p + (size_t)b * da.dt.sb * sizeof(T), (int)(da.dt.st * (long long)sizeof(T))};
    const Walked wz{(const char*)da.z.p + (size_t)b * da.z.sb * sizeof(T), (int)(da.z.st * (long long)sizeof(T))};
    const Walked wg{(const char*)a.dout.p + ((size_t)b * a.dout.sb + (a.separate ? s * a.Dn : 0)) * sizeof(T),
                    (int)(a.dout.st * (long long)sizeof(T))};
    const Walked wodx{(const char*)a.gdx[s].p + (size_t)b * a.gdx[s].sb * sizeof(T), (int)(a.gdx[s].st * (long long)sizeof(T))};
    const Walked wodz{(const char*)a.gdz[s].p + (size_t)b * a.gdz[s].sb * sizeof(T), (int)(a.gdz[s].st * (long long)sizeof(T))};
    const Walked woddt{(const char*)a.gddt[s].p + (size_t)b * a.gddt[s].sb * sizeof(T), (int)(a.gddt[s].st * (long long)sizeof(T))};
    const Walked wpk{(const char*)(a.parked + (size_t)b * a.L * a.Dn), a.Dn * (int)sizeof(Parked)};
    // this wave's slot of the dB | dC partial sums: [batch][L][G][slots][2N]
    const int tiles_per_group = (a.Dn / a.G + 63) / 64;
    const int slot = my_tile % tiles_per_group + (s == 1 ? a.bc_slot_of_rev : 0);
    const Walked wpart{(const char*)(a.bc_part[s] + (((size_t)b * a.L * a.G + grp) * a.bc_slots + slot) * (2 * N)),
                       a.G * a.bc_slots * 2 * N * (int)sizeof(float)};
    const Walked wrow{(const char*)c.bc, (int)(c.bcs * (long long)sizeof(float))};
    const char* const state_base = (const char*)(a.state + ((size_t)s * gridDim.z + b) * a.nchunk * a.Dn * N);
    const long long state_stride = (long long)a.Dn * N * (long long)sizeof(float);
    auto at_scan = [&](const Walked& t, int scan_index) { return t.base + (long long)c.token(scan_index) * t.stride; };
    // the per-token pointers start at the last token in scan order and move one token against it per step
    const char* p_odx = at_scan(wodx, a.L - 1);
    const char* p_odz = at_scan(wodz, a.L - 1);
    const char* p_oddt = at_scan(woddt, a.L - 1);
    const char* p_pk = at_scan(wpk, a.L - 1);
    const char* p_part = at_scan(wpart, a.L - 1);
    const char* p_row = at_scan(wrow, a.L - 1);
    const int s_odx = c.dir * wodx.stride, s_odz = c.dir * wodz.stride, s_oddt = c.dir * woddt.stride;
    const int s_pk = c.dir * wpk.stride, s_part = c.dir * wpart.stride, s_row = c.dir * wrow.stride;
    const int s_x = c.dir * wx.stride, s_dt = c.dir * wdt.stride, s_z = c.dir * wz.stride, s_g = c.dir * wg.stride;

    // In scan order both waves walk j = L-1 .. 0 and park j >= jm: tokens [L/2, L) for the forward direction's wave,
    // [0, L/2) for the reverse one's.  The other wave's values for j < jm are fetched two tokens ahead (q0, q1): a
    // load issued where its value is needed would stall the one wave this SIMD holds for a memory round trip.
    const int jm = a.park ? (s == 0 ? a.L / 2 : a.L - a.L / 2) : a.L;
    float q0[3] = {0.0f, 0.0f, 0.0f}, q1[3] = {0.0f, 0.0f, 0.0f};
    auto fetch_parked = [&](float (&q)[3], const char* row) {
        const Parked v = *(const Parked*)(row + lo_pk);
        q[0] = v.dx; q[1] = v.dz; q[2] = v.ddt;
    };
    // the barrier is a workgroup-scope release / acquire: past it, what the other wave of the tile parked is visible
    auto meet = [&]() {
        __syncthreads();
        if (jm >= 1) fetch_parked(q0, at_scan(wpk, jm - 1));
        if (jm >= 2) fetch_parked(q1, at_scan(wpk, jm - 2));
    };
    if (a.park && jm >= a.L) meet();                     // a one-token call: the reverse direction's wave parks nothing

    float dh[N], gA[N];
#pragma unroll
    for (int n = 0; n < N; n++) dh[n] = gA[n] = 0.0f;
    float gD = 0.0f, gcb = 0.0f, gbias = 0.0f, gw[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float dp1 = 0.0f, dp2 = 0.0f, dp3 = 0.0f;   // dpre of the tokens one, two, three steps later in scan order

    // as in the state pass: the next chunk's activations are requested before this chunk is worked through
    T xr[CT], dr[CT], zr[CT], gr[CT], xnext[CT], dnext[CT], znext[CT], gnext[CT];
    T xprev[3] = {};                                     // raw x of the three tokens before the chunk in xr
    float hnext[N];                                      // the state entering the next chunk to be walked
    auto request_state = [&](int k) {
        const float* src = (const float*)(state_base + k * state_stride + lo_state);
#pragma unroll
        for (int n = 0; n < N; n++) hnext[n] = src[n];
    };
    {   // the chunk walked first is the only one that can be short: its missing tokens repeat the last one
        const int k = a.nchunk - 1;
#pragma unroll
        for (int i = 0; i < CT; i++) {
            const int j = min(k * CT + i, a.L - 1);
            xr[i] = *(const T*)(at_scan(wx, j) + lo_t);
            dr[i] = *(const T*)(at_scan(wdt, j) + lo_t);
            zr[i] = *(const T*)(at_scan(wz, j) + lo_t);
            gr[i] = *(const T*)(at_scan(wg, j) + lo_t);
        }
        if (k > 0) {
#pragma unroll
            for (int e = 0; e < 3; e++) xprev[e] = *(const T*)(at_scan(wx, k * CT - 3 + e) + lo_t);
        }
        request_state(k);
    }
    for (int k = a.nchunk - 1; k >= 0; k--) {
        const int first = k * CT;                                   // scan index of the chunk's first token
        const int count = min(CT, a.L - first);
        keep_narrow(lo_t);
        keep_narrow(lo_pk);
        keep_narrow(lo_state);
        keep_narrow(lo_part);
        float xraw[CT + 3];
#pragma unroll
        for (int e = 0; e < 3; e++) xraw[e] = k > 0 ? IO::cvt(xprev[e]) : 0.0f;
        float hs[CT + 1][N];   // hs[i] = the state entering token i of the chunk
#pragma unroll
        for (int n = 0; n < N; n++) hs[0][n] = hnext[n];
        float xc[CT], delta[CT], pre[CT];
        // forward over the chunk, keeping every state
        const char* fwd_row = at_scan(wrow, first);
#pragma unroll
        for (int i = 0; i < CT; i++) {
            xraw[i + 3] = IO::cvt(xr[i]);
            pre[i] = fmaf(c.w4[0], xraw[i], fmaf(c.w4[1], xraw[i + 1], fmaf(c.w4[2], xraw[i + 2], fmaf(c.w4[3], xraw[i + 3], c.cb))));
            xc[i] = silu(pre[i]);
            delta[i] = c.delta_of(IO::cvt(dr[i]), sp);
            if (i < count) {
                const float u = delta[i] * xc[i];
                uniform_ro_ptr row = (uniform_ro_ptr)fwd_row;
#pragma unroll
                for (int n = 0; n < N; n++) hs[i + 1][n] = fmaf(fast_exp2(delta[i] * c.a2[n]), hs[i][n], u * row[n]);
            } else {
#pragma unroll
                for (int n = 0; n < N; n++) hs[i + 1][n] = hs[i][n];
            }
            fwd_row += s_row;
        }
        // backward over the chunk, last token first
#pragma unroll
        for (int i = CT - 1; i >= 0; i--) {
            // Half way through the walk the states of the chunk's later tokens are dead: their registers take the
            // next chunk (whole: one scalar step per tensor and token), its entering state and the three x before it.
            if (i == CT / 2 - 1 && k > 0) {
                const char* nx = at_scan(wx, first - CT);
                const char* nd = at_scan(wdt, first - CT);
                const char* nz = at_scan(wz, first - CT);
                const char* ng = at_scan(wg, first - CT);
                if (k > 1) {
#pragma unroll
                    for (int e = 0; e < 3; e++) xprev[e] = *(const T*)(nx - (3 - e) * (long long)s_x + lo_t);
                }
#pragma unroll
                for (int e = 0; e < CT; e++) {
                    xnext[e] = *(const T*)(nx + lo_t);
                    dnext[e] = *(const T*)(nd + lo_t);
                    znext[e] = *(const T*)(nz + lo_t);
                    gnext[e] = *(const T*)(ng + lo_t);
                    nx += s_x; nd += s_dt; nz += s_z; ng += s_g;
                }
                request_state(k - 1);
            }
            if (i >= count) continue;
            uniform_ro_ptr row = (uniform_ro_ptr)p_row;
            const float zv = IO::cvt(zr[i]);
            const float dg = valid ? IO::cvt(gr[i]) : 0.0f;          // shadow lanes add nothing to the sums below
            float y = c.dval * xc[i];
#pragma unroll
            for (int n = 0; n < N; n++) y = fmaf(row[N + n], hs[i + 1][n], y);
            const float dz = dg * y * dsilu(zv);
            const float dy = dg * silu(zv);
            gD = fmaf(dy, xc[i], gD);
            const float u_over = delta[i] * xc[i];
            float bc_terms[2 * N];                                   // this channel's terms of dB_t (first N) and dC_t
            // sum_n dh[n] B[n] serves both dDelta (times xc) and dxc (times Delta); sum_n (dh h_prev a)[n] a2[n] is
            // dDelta's decay part up to the factor ln 2 (A = a2 ln 2)
            float dh_dot_b = 0.0f, decay_part = 0.0f;
#pragma unroll
            for (int n = 0; n < N; n++) {
                const float an = fast_exp2(delta[i] * c.a2[n]);
                dh[n] = fmaf(row[N + n], dy, dh[n]);
                bc_terms[n] = dh[n] * u_over;
                bc_terms[N + n] = dy * hs[i + 1][n];
                const float da = dh[n] * hs[i][n] * an;              // dh * h_prev * a
                gA[n] = fmaf(da, delta[i], gA[n]);
                decay_part = fmaf(da, c.a2[n], decay_part);
                dh_dot_b = fmaf(dh[n], row[n], dh_dot_b);
                dh[n] *= an;
            }
            const float ddelta = fmaf(decay_part, kLn2, dh_dot_b * xc[i]);
            const float dxc = fmaf(c.dval, dy, dh_dot_b * delta[i]);
            {
                // the wave's 64 channels summed: value j ends up in lanes j * kLanesPerValue ..., one of which stores it
                const float total = wave_reduce_scatter<2 * N>(bc_terms, lane);
                if (exists && lane % kLanesPerValue == 0) *(float*)(const_cast<char*>(p_part) + lo_part) = total;
            }
            float ddt = ddelta;
            if (sp) {
                ddt *= sigmoidf(IO::cvt(dr[i]) + c.dtb);
                gbias += ddt;
            }
            const float dpre = dxc * dsilu(pre[i]);
            gcb += dpre;
            gw[3] = fmaf(dpre, xraw[i + 3], gw[3]);
            gw[2] = fmaf(dpre, xraw[i + 2], gw[2]);
            gw[1] = fmaf(dpre, xraw[i + 1], gw[1]);
            gw[0] = fmaf(dpre, xraw[i], gw[0]);
            const float dxv = fmaf(c.w4[3], dpre, fmaf(c.w4[2], dp1, fmaf(c.w4[1], dp2, c.w4[0] * dp3)));
            dp3 = dp2; dp2 = dp1; dp1 = dpre;
            const int j = first + i;
            if (j >= jm) {                                // never taken unless a.park
                if (valid) *(Parked*)(const_cast<char*>(p_pk) + lo_pk) = Parked{dxv, dz, ddt};
                if (j == jm) meet();
            } else {
                const float px = q0[0], pz = q0[1], pd = q0[2];
#pragma unroll
                for (int e = 0; e < 3; e++) q0[e] = q1[e];
                if (a.park && j >= 2) fetch_parked(q1, p_pk - 2 * (long long)s_pk);
                if (valid) {
                    IO::st((T*)(const_cast<char*>(p_odx) + lo_t), dxv + px);
                    IO::st((T*)(const_cast<char*>(p_odz) + lo_t), dz + pz);
                    IO::st((T*)(const_cast<char*>(p_oddt) + lo_t), ddt + pd);
                }
            }
            p_odx -= s_odx; p_odz -= s_odz; p_oddt -= s_oddt;
            p_pk -= s_pk; p_part -= s_part; p_row -= s_row;
        }
#pragma unroll
        for (int i = 0; i < CT; i++) {
            xr[i] = xnext[i];
            dr[i] = dnext[i];
            zr[i] = znext[i];
            gr[i] = gnext[i];
        }
    }
    if (valid) {
        const int K = a.K;
#pragma unroll
        for (int n = 0; n < N; n++) unsafeAtomicAdd(a.dA[s] + (size_t)ch * N + n, gA[n]);
        unsafeAtomicAdd(a.dD[s] + ch, gD);
#pragma unroll
        for (int i = 0; i < 4; i++)
            if (i < K) unsafeAtomicAdd(a.dconv_w[s] + (size_t)ch * K + (K - 1 - i), gw[3 - i]);
        if (a.dconv_b[s]) unsafeAtomicAdd(a.dconv_b[s] + ch, gcb);
        if (a.ddt_bias[s] && sp) unsafeAtomicAdd(a.ddt_bias[s] + ch, gbias);
    }
}

// dB and dC from the per-wave partial sums: one thread per (batch, token, group, value) adds its slots in a fixed order.
struct BwdBcArgs {
    const float* part;   // [batch][L][G][slots][2N]
    float* dB;           // [batch][L][G][N]
    float* dC;
    long long rows;      // batch * L * G
    int slots, N;
};

__global__ __launch_bounds__(256) void bwd_bc_kernel(const BwdBcArgs a);

}  // namespace bm
