// Device code of the bidirectional Mamba mixer path for gfx950 (CDNA4, wave64).
//
// Mapping: one lane owns one channel of one direction and walks the sequence token by token with its d_state
// recurrence values in registers; a wave covers 64 adjacent channels, so every per-token access of x / dt / z /
// out is one contiguous run.  B_t and C_t are wave-uniform and arrive through scalar loads from an fp32 copy made
// by prep_bc_kernel.  A workgroup holds the forward wave and the reverse wave of the same 64 channels.  For the
// additive combine (eq. 6) the two waves meet in the middle of the segment: in the first half of its walk each
// wave parks its gated output as an fp32 partial, in the second half it adds the partial the other wave parked
// there and performs the single rounding to the I/O dtype.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bm {

constexpr float kLog2e = 1.4426950408889634f;

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
};

struct IoF32 {
    using T = float;
    static __device__ __forceinline__ float ld(const T* p) { return *p; }
    static __device__ __forceinline__ float cvt(T v) { return v; }
    static __device__ __forceinline__ void st(T* p, float v) { *p = v; }
};
struct IoBF16 {
    using T = unsigned short;
    static __device__ __forceinline__ float cvt(T v) { return __uint_as_float(((unsigned)v) << 16); }
    static __device__ __forceinline__ float ld(const T* p) { return cvt(*p); }
    static __device__ __forceinline__ void st(T* p, float v)
    {
        __bf16 r = (__bf16)v;  // round to nearest even (v_cvt_pk_bf16_f32)
        *p = __builtin_bit_cast(unsigned short, r);
    }
};

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float silu(float v) { return v * __builtin_amdgcn_rcpf(1.0f + fast_exp2(-kLog2e * v)); }
__device__ __forceinline__ float softplus(float v) { return v > 20.0f ? v : log1pf(__expf(v)); }

enum { kSweep = 0, kSummary = 1 };
enum { kModePartial = 0, kModeFinalAdd = 1, kModeFinalOnly = 2, kModeNoOutput = 3 };

constexpr int kTile = 8;  // tokens whose loads are in flight while the previous tile is being computed

// Per-lane constants and running state of one (direction, channel) chain.
template <int N, int AKIND, typename IO>
struct Chain {
    using T = typename IO::T;
    float h[N];
    float a2[AKIND == 0 ? N : 1];  // A * log2(e)
    float w4[4];                   // conv taps, w4[3] on the current token
    float cb, dval, dtb, sum_dt;
    float xh[3];                   // previous raw x, xh[0] most recent
    const T *xp, *zp, *dtp;        // running pointers at the current token
    T* op;
    float* pp;                     // running pointer into the partial buffer
    uniform_ro_ptr bcp;            // uniform running pointer to this token's B|C row
    long long xs, zs, dts, os, ps, bcs;  // signed per-token steps in elements
};

template <int N, int AKIND, typename IO>
struct RawTile {
    typename IO::T x[kTile], z[kTile], dt[kTile];
    float part[kTile];
};

template <int N, int AKIND, typename IO, int MODE>
__device__ __forceinline__ void load_tile(const Chain<N, AKIND, IO>& c, RawTile<N, AKIND, IO>& r)
{
#pragma unroll
    for (int i = 0; i < kTile; i++) {
        r.x[i] = c.xp[i * c.xs];
        r.dt[i] = c.dtp[i * c.dts];
        if (MODE != kModeNoOutput) r.z[i] = c.zp[i * c.zs];
        if (MODE == kModeFinalAdd) r.part[i] = c.pp[i * c.ps];
    }
}

// One token of one chain: conv + SiLU, discretise, N state updates, skip term, gate, output.
template <int N, int AKIND, typename IO, int MODE>
__device__ __forceinline__ void token_step(Chain<N, AKIND, IO>& c, typename IO::T xraw, typename IO::T dtraw,
                                           typename IO::T zraw, float part, bool softplus_dt)
{
    const float x0 = IO::cvt(xraw);
    float pre = c.cb;
    pre = fmaf(c.w4[0], c.xh[2], pre);
    pre = fmaf(c.w4[1], c.xh[1], pre);
    pre = fmaf(c.w4[2], c.xh[0], pre);
    pre = fmaf(c.w4[3], x0, pre);
    c.xh[2] = c.xh[1];
    c.xh[1] = c.xh[0];
    c.xh[0] = x0;
    const float xc = silu(pre);
    float delta = IO::cvt(dtraw);
    if (softplus_dt) delta = softplus(delta + c.dtb);
    const float u = delta * xc;
    float y = c.dval * xc;
    uniform_ro_ptr bc = c.bcp;
    if (AKIND == 0) {
#pragma unroll
        for (int n = 0; n < N; n++) {
            const float a = fast_exp2(delta * c.a2[n]);
            c.h[n] = fmaf(a, c.h[n], u * bc[n]);
            if (MODE != kModeNoOutput) y = fmaf(bc[N + n], c.h[n], y);
        }
    } else {
        const float a = fast_exp2(delta * c.a2[0]);
#pragma unroll
        for (int n = 0; n < N; n++) {
            c.h[n] = fmaf(a, c.h[n], u * bc[n]);
            if (MODE != kModeNoOutput) y = fmaf(bc[N + n], c.h[n], y);
        }
    }
    if (MODE == kModeNoOutput) {
        c.sum_dt += delta;
    } else {
        const float g = y * silu(IO::cvt(zraw));
        if (MODE == kModePartial) {
            *c.pp = g;
        } else {
            const float o = MODE == kModeFinalAdd ? g + part : g;
            IO::st(c.op, o);
        }
    }
    c.xp += c.xs;
    c.dtp += c.dts;
    c.zp += c.zs;
    c.op += c.os;
    c.pp += c.ps;
    c.bcp += c.bcs;
}

// Tokens [0, count) of the chain's walk from its current position, tile by tile with the next tile's loads in flight.
template <int N, int AKIND, typename IO, int MODE>
__device__ __forceinline__ void run_range(Chain<N, AKIND, IO>& c, int count, bool softplus_dt)
{
    using Tile = RawTile<N, AKIND, IO>;
    int done = 0;
    if (count >= kTile) {
        Tile cur;
        load_tile<N, AKIND, IO, MODE>(c, cur);
        while (true) {
            const bool more = done + 2 * kTile <= count;
            Tile nxt;
            if (more) {
                // the next tile starts kTile tokens ahead of the running pointers
                Chain<N, AKIND, IO> ahead = c;
                ahead.xp += kTile * c.xs;
                ahead.dtp += kTile * c.dts;
                ahead.zp += kTile * c.zs;
                ahead.pp += kTile * c.ps;
                load_tile<N, AKIND, IO, MODE>(ahead, nxt);
            }
#pragma unroll
            for (int i = 0; i < kTile; i++)
                token_step<N, AKIND, IO, MODE>(c, cur.x[i], cur.dt[i], cur.z[i], cur.part[i], softplus_dt);
            done += kTile;
            if (!more) break;
            cur = nxt;
        }
    }
    for (; done < count; done++) {
        typename IO::T xr = *c.xp, dr = *c.dtp, zr = 0;
        float part = 0.0f;
        if (MODE != kModeNoOutput) zr = *c.zp;
        if (MODE == kModeFinalAdd) part = *c.pp;
        token_step<N, AKIND, IO, MODE>(c, xr, dr, zr, part, softplus_dt);
    }
}

// grid (ceil(Dn/64), nseg, batch), block 128: wave 0 walks left-to-right, wave 1 right-to-left.
template <int N, int AKIND, typename IO, int KIND>
__global__ __launch_bounds__(128) void sweep_kernel(const SweepArgs a)
{
    using T = typename IO::T;
    const int lane = threadIdx.x & 63;
    const int s = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const DirArgs& da = a.dir[s];
    const int b = blockIdx.z, seg = blockIdx.y;
    // Lanes past the last channel shadow channel Dn-1: they load the same inputs, compute the same values and
    // store them to the same addresses, so no lane needs masking anywhere below.
    const int ch = min((int)(blockIdx.x * 64 + lane), a.Dn - 1);
    const int head = ch / a.P;
    const int grp = (int)((blockIdx.x * 64) / a.P) / a.HG;  // uniform: a tile never straddles two B/C groups
    const int t0 = seg * a.seg_len;
    const int t1 = min(a.L, t0 + a.seg_len);
    const int len = t1 - t0;
    if (len <= 0) return;
    const int step = s == 0 ? 1 : -1;
    const int tstart = s == 0 ? t0 : t1 - 1;

    Chain<N, AKIND, IO> c;
    // per-lane constants
    {
        const int K = a.K;
#pragma unroll
        for (int i = 0; i < 4; i++) c.w4[3 - i] = i < K ? da.conv_w[(size_t)ch * K + (K - 1 - i)] : 0.0f;
        c.cb = da.conv_b ? da.conv_b[ch] : 0.0f;
        c.dval = da.D[a.d_per_head ? head : ch];
        c.dtb = (a.dt_softplus && da.dt_bias) ? da.dt_bias[head] : 0.0f;
        if (AKIND == 0) {
#pragma unroll
            for (int n = 0; n < N; n++) c.a2[n] = da.A[(size_t)head * N + n] * kLog2e;
        } else {
            c.a2[0] = da.A[head] * kLog2e;
        }
        c.sum_dt = 0.0f;
    }
    // initial state
    {
        const float* src = nullptr;
        if (KIND == kSweep) {
            if (a.nseg > 1) src = a.carry + ((((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch) * N;
            else if (s == 0 && a.h_in) src = a.h_in + ((size_t)b * a.Dn + ch) * N;
        }
#pragma unroll
        for (int n = 0; n < N; n++) c.h[n] = src ? src[n] : 0.0f;
    }
    // conv history: the K-1 raw tokens that precede the walk's first token in scan order
    {
        const T* xb = (const T*)da.x.p + (size_t)b * da.x.sb + ch;
#pragma unroll
        for (int i = 0; i < 3; i++) {
            const int t = tstart - step * (1 + i);
            float v = 0.0f;
            if (i < a.K - 1) {
                if (t >= 0 && t < a.L) v = IO::ld(xb + (long long)t * da.x.st);
                else if (t < 0 && s == 0 && a.tail_in)
                    v = IO::ld((const T*)a.tail_in + ((size_t)b * (a.K - 1) + (a.K - 1 + t)) * a.tail_ch + ch);
            }
            c.xh[i] = v;
        }
    }
    // running pointers and signed steps
    c.xs = step * da.x.st;
    c.zs = step * da.z.st;
    c.dts = step * da.dt.st;
    c.os = step * a.out_st;
    c.ps = step * (long long)a.Dn;
    c.bcs = step * (long long)(a.G * 2 * N);
    c.xp = (const T*)da.x.p + (size_t)b * da.x.sb + (long long)tstart * da.x.st + ch;
    c.zp = (const T*)da.z.p + (size_t)b * da.z.sb + (long long)tstart * da.z.st + ch;
    c.dtp = (const T*)da.dt.p + (size_t)b * da.dt.sb + (long long)tstart * da.dt.st + head;
    c.op = (T*)a.out + (size_t)b * a.out_sb + (long long)tstart * a.out_st + ch + (a.separate ? s * a.Dn : 0);
    c.pp = a.partial + ((size_t)b * a.L + tstart) * a.Dn + ch;
    c.bcp = (uniform_ro_ptr)(da.bc + (((size_t)b * a.L + tstart) * a.G + grp) * (2 * N));
    const bool sp = a.dt_softplus != 0;

    if (KIND == kSummary) {
        run_range<N, AKIND, IO, kModeNoOutput>(c, len, sp);
        {
            float* dst = a.carry + ((((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch) * N;
#pragma unroll
            for (int n = 0; n < N; n++) dst[n] = c.h[n];
            a.sumdt[(((size_t)s * gridDim.z + b) * a.nseg + seg) * a.Dn + ch] = c.sum_dt;
        }
        return;
    }

    if (a.separate) {
        run_range<N, AKIND, IO, kModeFinalOnly>(c, len, sp);
    } else {
        // forward parks [t0, m), reverse parks [m, t1); then each finishes the other's half
        const int n_first = s == 0 ? (len + 1) / 2 : len / 2;
        run_range<N, AKIND, IO, kModePartial>(c, n_first, sp);
        __syncthreads();  // workgroup-scope release/acquire: the other wave's partials are visible from here on
        run_range<N, AKIND, IO, kModeFinalAdd>(c, len - n_first, sp);
    }
    if (s == 0 && a.nseg == 1 && a.h_out) {
        float* dst = a.h_out + ((size_t)b * a.Dn + ch) * N;
#pragma unroll
        for (int n = 0; n < N; n++) dst[n] = c.h[n];
    }
}

// Stitch time segments: carry[s][b][seg] holds each segment's end state from a zero start (summary pass); replace it
// by the state entering the segment, folding (decay product, end state) pairs in scan order:
//   h_next = exp(A * sum_dt_seg) * h + S_seg.      One thread per (direction, batch, channel).
struct CarryArgs {
    float* carry;
    const float* sumdt;
    const float* A[2];
    const float* h_in;
    float* h_out;
    int batch, nseg, Dn, P;
};

template <int N, int AKIND>
__global__ __launch_bounds__(256) void carry_kernel(const CarryArgs a)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = 2LL * a.batch * a.Dn;
    if (idx >= total) return;
    const int ch = (int)(idx % a.Dn);
    const int b = (int)((idx / a.Dn) % a.batch);
    const int s = (int)(idx / ((long long)a.Dn * a.batch));
    const int head = ch / a.P;
    float a2[AKIND == 0 ? N : 1];
    if (AKIND == 0) {
#pragma unroll
        for (int n = 0; n < N; n++) a2[n] = a.A[s][(size_t)head * N + n] * kLog2e;
    } else {
        a2[0] = a.A[s][head] * kLog2e;
    }
    float h[N];
    const float* hin = (s == 0 && a.h_in) ? a.h_in + ((size_t)b * a.Dn + ch) * N : nullptr;
#pragma unroll
    for (int n = 0; n < N; n++) h[n] = hin ? hin[n] : 0.0f;
    for (int i = 0; i < a.nseg; i++) {
        const int seg = s == 0 ? i : a.nseg - 1 - i;
        const size_t row = (((size_t)s * a.batch + b) * a.nseg + seg) * a.Dn + ch;
        float* S = a.carry + row * N;
        const float sd = a.sumdt[row];
#pragma unroll
        for (int n = 0; n < N; n++) {
            const float end_state = S[n];
            S[n] = h[n];
            const float p = fast_exp2(sd * a2[AKIND == 0 ? n : 0]);
            h[n] = fmaf(p, h[n], end_state);
        }
    }
    if (s == 0 && a.h_out) {
        float* dst = a.h_out + ((size_t)b * a.Dn + ch) * N;
#pragma unroll
        for (int n = 0; n < N; n++) dst[n] = h[n];
    }
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
