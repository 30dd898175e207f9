// Chunked state-space-duality kernels for the Mamba-2 parameterisation (one decay rate per head) on gfx950.
//
// With a scalar decay per head the recurrence over a chunk of Q = 64 tokens is a set of dense contractions
// (j, i: positions in the chunk in scan order; l_i = sum_{r<=i} Delta_r A; H: state entering the chunk, [N, P]):
//   y_i   = sum_{j<=i} (C_i . B_j) exp(l_i - l_j) Delta_j xc_j  +  exp(l_i) C_i H  +  D xc_i
//   H_out = exp(l_Q) H + sum_j exp(l_Q - l_j) Delta_j B_j^T xc_j
// which run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).  One workgroup owns one
// (direction, batch, head) and walks the chunks in scan order with H in accumulator registers (fp32 for the whole
// sequence).  Decay factors are formed in fp32; only MFMA operands (xc, B, C, the masked score tile, a copy of H) are
// rounded to bf16.  ssd_prep_kernel builds, once per (direction, batch, chunk, group) and shared by all heads, the
// score tile C B^T, the bf16 C rows and the transposed bf16 B tile.
//
// Kernels in this file: ssd_prep_kernel (above); ssd_kernel, the chunk walk of one direction (ssd_walk), with
// variants for two producer groups and for time parts; ssd_state_kernel and ssd_carry_kernel, which find the state
// entering each time part when a call has too few (batch, head) items to fill the chip; ssd_duo_kernel, both
// directions of a single-chunk call (a block-diffusion step) in one workgroup.
//
// Lane layouts of the 32x32x16 MFMA (checked on hardware): operand A lane l holds row l%32, k = 8*(l/32)..+7;
// operand B lane l holds column l%32, same k; accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
// column l%32.  A contraction index may be enumerated in any order as long as both operands agree, which lets an
// accumulator tile be fed back as an operand without a transpose: registers 8*kb..8*kb+7 of a lane are the 8
// k-slots of k-block kb, i.e. k = 16*kb + 8*jj + 4*(l/32) + e for slot 4*jj + e.
#pragma once
#include "kernels.h"
#include <type_traits>

namespace bm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kQ = 64;     // chunk length
constexpr int kPadK = 8;   // bf16 elements of row padding in LDS tiles (keeps 16-byte alignment, spreads banks)
constexpr int kScoreOp = 3 * 2 * 64 * 8;   // floats of one chunk's score tile: 3 lower-triangular 32x32 blocks

struct SsdPrepArgs {
    TensorArg B, C;       // bf16 [batch][L][G*N]
    const float* conv_w;  // full [conv_ch][K] table of this direction (rows Dn.. are B|C) when conv_bc
    const float* conv_b;  // or null
    const void* tail_in;  // bf16 [batch][K-1][tail_ch] or null (causal direction of the block variant)
    __bf16* c_rows;    // [batch][Lpad][G][N], scan order
    __bf16* b_t;       // [batch][nchunk][G][N][64], scan order inside the chunk
    float* score_op;   // [batch][nchunk][G][kScoreOp]: B_j . C_i for j, i in the chunk, MFMA operand order (see the kernel)
    int L, G, K, Dn, tail_ch, conv_bc;
    int dir;           // +1: scan position tau is token tau; -1: token L-1-tau
};

struct SsdPrepPair {
    SsdPrepArgs dir[2];   // forward, reverse: one launch prepares both
};

// (the wide form adds the partial score accumulators of the waves that share a block: [12][64][16] floats)
template <int N, int THREADS>
constexpr size_t ssd_prep_lds_bytes()
{
    return 2 * (size_t)kQ * (N + 1) * sizeof(float) + (THREADS > 256 ? 12 * 64 * 16 * sizeof(float) : 0);
}

// grid (nchunk, G, 2 * batch), block THREADS (256 or 1024), dynamic LDS ssd_prep_lds_bytes<N, THREADS>();
// blockIdx.z / batch selects the direction.  Reads the raw B and C rows of one chunk
// (plus the conv halo), applies the short conv + SiLU along the scan direction when they pass through it, and
// keeps the fp32 result in LDS for the three outputs.  The wide form is for launches of few workgroups (block
// calls, short sequences), whose duration is one workgroup's chain of phases: sixteen waves shorten every phase.
template <int N, int THREADS = 256>
__global__ __launch_bounds__(THREADS) void ssd_prep_kernel(const SsdPrepPair both)
{
    static_assert(THREADS == 256 || THREADS == 1024, "four or sixteen waves");
    using T = unsigned short;
    const int batch = gridDim.z / 2;
    const SsdPrepArgs& a = both.dir[blockIdx.z / batch];
    extern __shared__ __attribute__((aligned(16))) unsigned char ssd_prep_lds[];
    float(*sB)[N + 1] = reinterpret_cast<float(*)[N + 1]>(ssd_prep_lds);
    float(*sC)[N + 1] = sB + kQ;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z % batch, tid = threadIdx.x;
    const int nchunk = gridDim.x;
    {
        constexpr int kCols = 2 * N, kParts = THREADS / kCols, kLen = kQ / kParts;
        const int col = tid % kCols, seg = tid / kCols;   // one column of B|C, positions seg*kLen .. of the chunk
        const int which = col / N, n = col % N;
        const TensorArg& src = which ? a.C : a.B;
        const T* base = (const T*)src.p + (size_t)b * src.sb + g * N + n;
        const int last = a.L - 1;
        const int row = a.Dn + which * a.G * N + g * N + n;   // this column's conv channel
        float w4[4] = {0.0f, 0.0f, 0.0f, 0.0f}, bias = 0.0f;   // w4[3] on the current position
        if (a.conv_bc) {
#pragma unroll
            for (int i = 0; i < 4; i++) w4[3 - i] = i < a.K ? a.conv_w[(size_t)row * a.K + (a.K - 1 - i)] : 0.0f;
            bias = a.conv_b ? a.conv_b[row] : 0.0f;
        }
        const int tau0 = c * kQ + seg * kLen - 3;
        T raw[kLen + 3];
#pragma unroll
        for (int q = 0; q < kLen + 3; q++) {
            const int tau = min(max(tau0 + q, 0), last);
            raw[q] = base[(long long)(a.dir > 0 ? tau : last - tau) * src.st];
        }
        float xr[kLen + 3];
#pragma unroll
        for (int q = 0; q < kLen + 3; q++) xr[q] = (tau0 + q >= 0 && tau0 + q <= last) ? IoBF16::cvt(raw[q]) : 0.0f;
        if (c == 0 && seg == 0 && a.dir > 0 && a.tail_in && a.conv_bc && a.K > 1) {
            // requested together from clamped rows (a tap beyond the conv width has a zero weight)
            T cached[3];
#pragma unroll
            for (int q = 0; q < 3; q++)   // 3 - q tokens before the block
                cached[q] = ((const T*)a.tail_in)[((size_t)b * (a.K - 1) + max(a.K - 1 - (3 - q), 0)) * a.tail_ch + row];
#pragma unroll
            for (int q = 0; q < 3; q++)
                if (3 - q <= a.K - 1) xr[q] = IoBF16::cvt(cached[q]);
        }
        float(*dstm)[N + 1] = which ? sC : sB;
#pragma unroll
        for (int i = 0; i < kLen; i++) {
            float v = xr[i + 3];
            if (a.conv_bc) {
                float pre = bias;
                pre = fmaf(w4[0], xr[i], pre);
                pre = fmaf(w4[1], xr[i + 1], pre);
                pre = fmaf(w4[2], xr[i + 2], pre);
                pre = fmaf(w4[3], xr[i + 3], pre);
                v = silu(pre);
            }
            if (tau0 + 3 + i > last) v = 0.0f;
            dstm[seg * kLen + i][n] = v;
        }
    }
    __syncthreads();
    const size_t Lpad = (size_t)nchunk * kQ;
    // bf16 C rows and the transposed bf16 B tile, written as 16-byte pieces (8 states of a row, 8 positions of a state)
    for (int idx = tid; idx < kQ * N / 8; idx += THREADS) {
        const int j = idx / (N / 8), n8 = idx % (N / 8);
        const int n2 = idx / (kQ / 8), j8 = idx % (kQ / 8);
        bf16x8 cv, bv;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            cv[e] = (__bf16)sC[j][8 * n8 + e];
            bv[e] = (__bf16)sB[8 * j8 + e][n2];
        }
        *reinterpret_cast<bf16x8*>(&a.c_rows[(((size_t)b * Lpad + c * kQ + j) * a.G + g) * N + 8 * n8]) = cv;
        *reinterpret_cast<bf16x8*>(&a.b_t[((((size_t)b * nchunk + c) * a.G + g) * N + n2) * kQ + 8 * j8]) = bv;
    }
    // Score tile B_j . C_i on the matrix cores, one 32 x 32 block per wave; only the three blocks on or below the
    // diagonal are kept.  Each fp32 operand is split into a bf16 head and a bf16 remainder and the three significant
    // cross products are accumulated in fp32, which keeps about 16 bits of the products.  With B rows as operand A
    // and C rows as operand B, accumulator register r of lane l is row j%32 = 8*(r/4) + 4*(l/32) + r%4 of column
    // i%32 = l%32: exactly the order in which the scan kernel feeds the tile to its MFMA as operand A,
    // [block pair (0,0), (1,0), (1,1)][k-block r/8][lane][r%8].
    const int wave = tid / 64, lane = tid % 64;
    // The wide form deals a block's N / 16 contraction steps to four waves and adds their accumulators through LDS.
    constexpr int kSplit = THREADS > 256 ? 4 : 1;
    constexpr int kSteps = N / 16 / kSplit;
    const int blk = wave / kSplit, kpart = wave % kSplit;
    f32x16 acc = {0};
    if (blk < 3) {
        const int iblk = blk > 0, jblk = blk > 1;
        const int rj = jblk * 32 + lane % 32, ri = iblk * 32 + lane % 32, koff = 8 * (lane / 32);
        for (int ks = kpart * kSteps; ks < (kpart + 1) * kSteps; ks++) {
            bf16x8 ah, al, bh, bl;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const float bv = sB[rj][16 * ks + koff + e], cv = sC[ri][16 * ks + koff + e];
                ah[e] = (__bf16)bv;
                al[e] = (__bf16)(bv - (float)ah[e]);
                bh[e] = (__bf16)cv;
                bl[e] = (__bf16)(cv - (float)bh[e]);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
        }
    }
    if constexpr (kSplit > 1) {
        float* const sums = reinterpret_cast<float*>(sC + kQ);   // [12][64][16]
        if (blk < 3 && kpart > 0) {
#pragma unroll
            for (int q = 0; q < 4; q++)
                *reinterpret_cast<float4*>(&sums[((size_t)wave * 64 + lane) * 16 + 4 * q]) =
                    make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        }
        __syncthreads();
        if (blk < 3 && kpart == 0) {
            for (int o = 1; o < kSplit; o++) {
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float4 v = *reinterpret_cast<const float4*>(&sums[((size_t)(wave + o) * 64 + lane) * 16 + 4 * q]);
                    acc[4 * q] += v.x; acc[4 * q + 1] += v.y; acc[4 * q + 2] += v.z; acc[4 * q + 3] += v.w;
                }
            }
        }
    }
    if (blk < 3 && kpart == 0) {
        float* dst = a.score_op + (((size_t)b * nchunk + c) * a.G + g) * kScoreOp + ((size_t)(blk * 2) * 64 + lane) * 8;
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
            *reinterpret_cast<float4*>(dst + kb * 64 * 8) = make_float4(acc[8 * kb], acc[8 * kb + 1], acc[8 * kb + 2], acc[8 * kb + 3]);
            *reinterpret_cast<float4*>(dst + kb * 64 * 8 + 4) = make_float4(acc[8 * kb + 4], acc[8 * kb + 5], acc[8 * kb + 6], acc[8 * kb + 7]);
        }
    }
}

// Output modes of ssd_kernel.
enum { kSsdFinalOnly = 0, kSsdPartial = 1, kSsdPartialRaw = 2, kSsdFinalAdd = 3, kSsdFinalAddRaw = 4 };

struct SsdArgs {
    TensorArg x, z, dt;
    const float *conv_w, *conv_b, *A, *D, *dt_bias;
    const __bf16* c_rows;
    const __bf16* b_t;
    const float* score_op;
    void* out;
    long long out_sb, out_st;
    float* partial;       // [batch][L][Dn] fp32
    const float* h_in;    // [batch][Dn][N] or null
    float* h_out;         // or null
    const void* tail_in;  // bf16 [batch][K-1][tail_ch] or null (causal direction only)
    int L, Dn, H, HG, G, K, tail_ch, nchunk;
    int dir, mode, out_ch_off, dt_softplus, d_per_head;
    int wide;             // run on ssd_wide_kernel (ssd_wide.h): both directions of a call agree, the parked result is bf16
    // Time parts (calls with too few (batch, head) items to fill the chip): the chunks are dealt to `parts` workgroups
    // per item, part_chunks each, in scan order (blockIdx.y).  A part is part_subs sub-parts of sub_chunks chunks;
    // ssd_state_kernel leaves every sub-part's end state from a zero start and the product of its chunk decays (all
    // but the scan-last one), ssd_carry_kernel turns those into the state entering each sub-part, and the output launch
    // starts part p from the entry state of sub-part p * part_subs.
    int parts, part_chunks, part_subs, sub_chunks;
    float* part_state;    // [subs][batch][Dn][N]
    float* part_decay;    // [subs][batch][H]
};

struct SsdCarryArgs {
    float* part_state[2];
    const float* part_decay[2];
    const float* h_in;    // forward direction's initial state or null
    int batch, Dn, P, H, parts;   // parts: the number of sub-parts to fold over
};

// One thread per (direction, batch, channel, four states): entry state of sub-part p+1 = decay_p * entry_p + end_p.
template <int N>
__global__ __launch_bounds__(256) void ssd_carry_kernel(const SsdCarryArgs a)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long per_dir = (long long)a.batch * a.Dn * N / 4;
    if (idx >= 2 * per_dir) return;
    const int s = (int)(idx / per_dir);
    const long long e = (idx % per_dir) * 4;            // element offset inside one part's [batch][Dn][N]
    const int ch = (int)((e / N) % a.Dn), b = (int)(e / ((long long)N * a.Dn));
    float4 h = (s == 0 && a.h_in) ? *reinterpret_cast<const float4*>(a.h_in + e) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = 0; p < a.parts; p++) {
        float4* slot = reinterpret_cast<float4*>(a.part_state[s] + (size_t)p * per_dir * 4 + e);
        const bool more = p + 1 < a.parts;
        const float4 end = more ? *slot : make_float4(0.f, 0.f, 0.f, 0.f);
        *slot = h;
        if (more) {
            const float dk = a.part_decay[s][((size_t)p * a.batch + b) * a.H + ch / a.P];
            h = make_float4(fmaf(dk, h.x, end.x), fmaf(dk, h.y, end.y), fmaf(dk, h.z, end.z), fmaf(dk, h.w, end.w));
        }
    }
}

// LDS of ssd_kernel: two buffers of per-chunk tiles (filled by the producer waves one chunk ahead of the consumer
// waves) and two copies of the state in MFMA operand form.  SINGLE (calls of one chunk, i.e. block-diffusion steps):
// one of each and one set of scan tables shared by the producer waves (they all write the same values), which brings
// the workgroup under half a CU's LDS so that two workgroups overlap their load-compute-store chains on a CU.
template <int N, int P, bool SINGLE = false>
struct SsdLds {
    static constexpr int kRowC = N + kPadK, kRowT = kQ + kPadK;
    static constexpr int kC = kQ * kRowC;    // C rows of the chunk               [kQ][kRowC] bf16
    static constexpr int kBT = N * kRowT;    // B transposed                      [N][kRowT]  bf16
    static constexpr int kX = P * kRowT;     // conv + SiLU output, transposed    [P][kRowT]  bf16 (two of them)
    static constexpr int kM = 2 * 2 * 2 * 64 * 8;   // masked, decayed score tile as MFMA operands [iblk][jblk][kb][lane][8]
    static constexpr int kTileElems = kC + kBT + 2 * kX + kM;
    static constexpr int kHT = (N / 32) * (P / 32) * 2 * 64 * 8;   // state operand copy, bf16
    static constexpr int kProducerWaves = 4;
    static constexpr int kBufs = SINGLE ? 1 : 2;
    static constexpr int kScanTables = SINGLE ? 1 : kProducerWaves;
    // + exp(l_i) per buffer, + per scan table: cumulative log2 decay, Delta, end-of-chunk weight of each position
    static constexpr size_t bytes() { return (size_t)(kBufs * kTileElems + kBufs * kHT) * sizeof(__bf16) + (kBufs + 3 * kScanTables) * kQ * sizeof(float); }
};

// LDS-only barrier: waits for this wave's LDS traffic, not for global loads that were issued ahead on purpose.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Inclusive prefix sum over the 64 lanes with DPP moves: shifts inside each row of 16 lanes, then the last lane of
// row 0 / 2 is added to row 1 / 3 and the last lane of row 1 to rows 2 and 3.
__device__ __forceinline__ float wave_inclusive_sum(float v)
{
#define BM_DPP_ADD(ctrl, rows) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rows, 0xF, false))
    BM_DPP_ADD(0x111, 0xF);  // row_shr:1
    BM_DPP_ADD(0x112, 0xF);  // row_shr:2
    BM_DPP_ADD(0x114, 0xF);  // row_shr:4
    BM_DPP_ADD(0x118, 0xF);  // row_shr:8
    BM_DPP_ADD(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
    BM_DPP_ADD(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef BM_DPP_ADD
    return v;
}

struct SsdStatePair {
    SsdArgs dir[2];   // forward, reverse: one launch walks both
};

// State pass of the time parts.  grid (H, subs - 1, 2 * batch), block 256, static LDS; blockIdx.z / batch selects the
// direction and blockIdx.y the sub-part: sub_chunks chunks in scan order, walked from a zero state.  Leaves the
// sub-part's end state in part_state[sub] and the product of its chunk decays in part_decay[sub] for
// ssd_carry_kernel.  The end state needs neither the score tile nor C nor the gate, so this is the conv + SiLU of x,
// the chunk's decay weights and the state-update product only, in a workgroup light enough (four waves, 19 KB of LDS)
// that three or four of them share a CU; the sub-parts are what gives the chip that many workgroups.  All four
// waves run the short scan for themselves, convolve a quarter of the chunk's positions each, and own 1/4 of the
// 32 x 32 blocks of H, whose B^T operand they read straight from the prepared tile in global memory.
template <int N, int P>
__global__ __launch_bounds__(256, 4) void ssd_state_kernel(const SsdStatePair both)
{
    constexpr int kPB = P / 32, kNB = N / 32, kBlocks = kNB * kPB, kOwn = (kBlocks + 3) / 4;
    constexpr int kRowT = kQ + kPadK;
    constexpr int kCP = P / 2;                // channel pairs of the head
    constexpr int kPos = kQ * kCP / 256;      // chunk positions per thread in the conv (8 or 4)
    using T = unsigned short;
    __shared__ __attribute__((aligned(16))) __bf16 s_xw[2][P * kRowT];   // conv output times end-of-chunk weight, transposed
    __shared__ __attribute__((aligned(16))) float s_wgt[4][kQ];          // wave-private: end-of-chunk weight of each position

    // (a compare, not a division by the batch size: integer division runs on the vector ALU)
    const int batch = gridDim.z >> 1;
    const int reverse = (int)blockIdx.z >= batch ? 1 : 0;
    const SsdArgs& a = both.dir[reverse];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int head = blockIdx.x, b = (int)blockIdx.z - reverse * batch, sub = blockIdx.y;
    const int grp = head / a.HG, ch0 = head * P;
    // (the host never hands this pass the sequence's last sub-part, so every chunk here is a full one)
    const int c_first = sub * a.sub_chunks, c_stop = min(a.L / kQ, c_first + a.sub_chunks);
    const int last = a.L - 1;
    auto token_of = [&](int tau) { return a.dir > 0 ? tau : last - tau; };

    const int cp = tid % kCP, tg = tid / kCP;   // conv role: channels 2cp, 2cp+1; positions kPos*tg .. of each chunk
    const float a2 = a.A[head] * kLog2e;
    const float dtb = (a.dt_softplus && a.dt_bias) ? a.dt_bias[head] : 0.0f;
    float w4[2][4], cbias[2];
#pragma unroll
    for (int h2 = 0; h2 < 2; h2++) {
#pragma unroll
        for (int i = 0; i < 4; i++)
            w4[h2][3 - i] = i < a.K ? a.conv_w[(size_t)(ch0 + 2 * cp + h2) * a.K + (a.K - 1 - i)] : 0.0f;
        cbias[h2] = a.conv_b ? a.conv_b[ch0 + 2 * cp + h2] : 0.0f;
    }
    const T* xb = (const T*)a.x.p + (size_t)b * a.x.sb + ch0 + 2 * cp;
    const T* dtp = (const T*)a.dt.p + (size_t)b * a.dt.sb + head;
    float* const wgt = s_wgt[wave];

    // matrix role: blocks kOwn * wave + o of the kNB x kPB blocks of H, channel block fastest, so that the blocks of a
    // wave share their rows of B^T (kSameB: one operand load serves both)
    constexpr bool kSameB = kOwn == 2 && kPB == 2;
    constexpr int kLoadB = kSameB ? 1 : kOwn;
    const int cl = lane & 31, half = lane >> 5;
    f32x16 hacc[kOwn];
#pragma unroll
    for (int o = 0; o < kOwn; o++)
#pragma unroll
        for (int r = 0; r < 16; r++) hacc[o][r] = 0.0f;

    // channel pair at positions kPos*tg - 3 .. kPos*tg + kPos - 1 and Delta of position `lane`, as requested for the
    // chunk after the one being worked on
    unsigned xnext[kPos + 3];
    T dtraw;
    auto issue_dt = [&](int c) { dtraw = dtp[(long long)token_of(min(c * kQ + lane, last)) * a.dt.st]; };
    // A chunk inside the sequence is read through a raw buffer range anchored at the chunk's lowest token row: the
    // row of register q is a wave-uniform offset, the thread's rows and channel pair a 32-bit offset that never
    // changes (no per-row vector address arithmetic, no address registers).  The host keeps 67 rows within 2^32 bytes.
    const unsigned st_bytes = (unsigned)a.x.st * (unsigned)sizeof(T);
    const unsigned x_lane_off = (unsigned)(a.dir > 0 ? kPos * tg : kQ - kPos * (tg + 1)) * st_bytes + 4u * cp;
    const T* const x_head = (const T*)a.x.p + (size_t)b * a.x.sb + ch0;
    auto issue_x_inside = [&](int c) {   // chunks 1 .. L / kQ - 1
        {
            const Rsrc rows = raw_range(x_head + (long long)(a.dir > 0 ? c * kQ - 3 : last - (c * kQ + kQ - 1)) * a.x.st);
            // register q holds scan position q of the thread, so the rows run backwards in the reverse direction.
            // (The offsets are formed in scalar registers for every chunk anew: carried across the loop, the compiler
            // keeps them in vector registers and loops over the lanes to read them back for each load.)
            int row_step = __builtin_amdgcn_readfirstlane(a.dir * (int)st_bytes);
            asm volatile("" : "+s"(row_step));
            const int row_0 = ((1 - a.dir) >> 1) * (kPos + 2) * (a.dir * row_step);
#pragma unroll
            for (int q = 0; q < kPos + 3; q++)
                xnext[q] = __builtin_amdgcn_raw_buffer_load_b32(rows, x_lane_off, row_0 + q * row_step, 0);
        }
    };
    auto issue_x_first = [&]() {   // chunk 0: positions before the sequence are clamped here and zeroed in the conv
        const int tau0 = kPos * tg - 3;
#pragma unroll
        for (int q = 0; q < kPos + 3; q++)
            xnext[q] = *reinterpret_cast<const unsigned*>(xb + (long long)token_of(min(max(tau0 + q, 0), last)) * a.x.st);
    };
    if (c_first >= c_stop) return;   // (never: see above)
    issue_dt(c_first);
    if (c_first == 0) issue_x_first(); else issue_x_inside(c_first);
    float decay_product = 1.0f;
    // The walk is bound by the latency of its loads (a row piece of 128 bytes per token, each from another DRAM page),
    // not by its arithmetic: what chunk c + 1 needs is requested at the top of chunk c, a whole chunk of work ahead,
    // and on every path alike (the walk's last chunk re-requests a valid chunk), so that the waits below count the
    // same loads in flight whichever way the loop was entered.
    const int c_inside = a.L / kQ - 1;   // the last chunk that is certainly a full one
    for (int c = c_first; c < c_stop; c++) {
        const int buf = (c - c_first) & 1;
        const int cn = max(1, min(c + 1, c_inside));
        // take over what was requested for this chunk
        unsigned xraw[kPos + 3];
#pragma unroll
        for (int q = 0; q < kPos + 3; q++) xraw[q] = xnext[q];
        float dl = IoBF16::cvt(dtraw);
        issue_dt(cn);
        // this wave's B^T operands straight from the prepared tile (rows of kQ positions), used after the barrier.
        bf16x8 ab[kLoadB][4];
        {
            const __bf16* bsrc = a.b_t + ((((size_t)b * a.nchunk + c) * a.G + grp) * N) * kQ;
#pragma unroll
            for (int o = 0; o < kLoadB; o++) {
                const int id = kOwn * wave + o, nblk = id / kPB;
                if (kBlocks % 4 == 0 || id < kBlocks) {
#pragma unroll
                    for (int kb = 0; kb < 4; kb++)
                        ab[o][kb] = *reinterpret_cast<const bf16x8*>(bsrc + (nblk * 32 + cl) * kQ + 16 * kb + 8 * half);
                }
            }
        }
        issue_x_inside(cn);
        // Delta, inclusive cumulative log2-decay, end-of-chunk weight of position `lane`
        if (a.dt_softplus) dl = softplus(dl + dtb);
        if (c * kQ + lane > last) dl = 0.0f;
        const float l2 = wave_inclusive_sum(dl * a2);
        const float l2_end = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 63));
        wgt[lane] = fast_exp2(l2_end - l2) * dl;
        const float decay_q = fast_exp2(l2_end);
        __builtin_amdgcn_wave_barrier();
        // conv + SiLU of two channels at kPos positions, weighted
        if (c == 0) {
#pragma unroll
            for (int q = 0; q < 3; q++)
                if (kPos * tg + q - 3 < 0) xraw[q] = 0u;
            if (a.dir > 0 && a.tail_in && tg == 0 && a.K > 1) {
                unsigned cached[3];
#pragma unroll
                for (int q = 0; q < 3; q++) {   // 3 - q tokens before the block (a tap beyond the conv width has a zero weight)
                    const T* tp = (const T*)a.tail_in + ((size_t)b * (a.K - 1) + max(a.K - 1 - (3 - q), 0)) * a.tail_ch + ch0 + 2 * cp;
                    cached[q] = (unsigned)tp[0] | ((unsigned)tp[1] << 16);
                }
                // (consumed here, so that no load is pending on xraw where the two paths join: the conv must not
                // wait for the younger B^T loads)
#pragma unroll
                for (int q = 0; q < 3; q++) asm volatile("" : "+v"(cached[q]));
#pragma unroll
                for (int q = 0; q < 3; q++)
                    if (3 - q <= a.K - 1) xraw[q] = cached[q];
            }
        }
        float wq[kPos];
#pragma unroll
        for (int q = 0; q < kPos; q += 4) {
            const float4 w = *reinterpret_cast<const float4*>(&wgt[kPos * tg + q]);
            wq[q] = w.x; wq[q + 1] = w.y; wq[q + 2] = w.z; wq[q + 3] = w.w;
        }
#pragma unroll
        for (int h2 = 0; h2 < 2; h2++) {
            typedef __attribute__((__vector_size__(kPos * sizeof(__bf16)))) __bf16 bf16run;
            float xr[kPos + 3];
#pragma unroll
            for (int q = 0; q < kPos + 3; q++) xr[q] = __uint_as_float(h2 == 0 ? xraw[q] << 16 : xraw[q] & 0xffff0000u);
            bf16run vw;
#pragma unroll
            for (int q = 0; q < kPos; q++) {
                float pre = cbias[h2];
                pre = fmaf(w4[h2][0], xr[q], pre);
                pre = fmaf(w4[h2][1], xr[q + 1], pre);
                pre = fmaf(w4[h2][2], xr[q + 2], pre);
                pre = fmaf(w4[h2][3], xr[q + 3], pre);
                vw[q] = (__bf16)(silu(pre) * wq[q]);
            }
            *reinterpret_cast<bf16run*>(&s_xw[buf][(2 * cp + h2) * kRowT + kPos * tg]) = vw;
        }
        lds_barrier();   // one per chunk: the other buffer is rewritten only after every wave has passed this one
        decay_product *= decay_q;
#pragma unroll
        for (int o = 0; o < kOwn; o++) {
            const int id = kOwn * wave + o, pblk = id % kPB;
            if (kBlocks % 4 == 0 || id < kBlocks) {
#pragma unroll
                for (int r = 0; r < 16; r++) hacc[o][r] *= decay_q;
#pragma unroll
                for (int kb = 0; kb < 4; kb++) {
                    const bf16x8 bw = *reinterpret_cast<const bf16x8*>(&s_xw[buf][(pblk * 32 + cl) * kRowT + 16 * kb + 8 * half]);
                    hacc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab[kSameB ? 0 : o][kb], bw, hacc[o], 0, 0, 0);
                }
            }
        }
    }
    if (tid == 0) a.part_decay[((size_t)sub * batch + b) * a.H + head] = decay_product;
    float* const state_out = a.part_state + (size_t)sub * batch * a.Dn * N;
#pragma unroll
    for (int o = 0; o < kOwn; o++) {
        const int id = kOwn * wave + o, nblk = id / kPB, pblk = id % kPB;
        if (kBlocks % 4 == 0 || id < kBlocks) {
            // registers 4q .. 4q+3 hold four adjacent states of channel pblk*32 + cl
            float* hrow = state_out + ((size_t)b * a.Dn + ch0 + pblk * 32 + cl) * N + nblk * 32 + 4 * half;
#pragma unroll
            for (int q = 0; q < 4; q++)
                *reinterpret_cast<float4*>(hrow + 8 * q) =
                    make_float4(hacc[o][4 * q], hacc[o][4 * q + 1], hacc[o][4 * q + 2], hacc[o][4 * q + 3]);
        }
    }
}

// grid (H, 1, batch), block 4*P + 256, dynamic LDS SsdLds<N, P>::bytes().  x is read as pairs of channels: its pointer
// must be 4-byte aligned and its strides even (the host checks).
// The first P/16 waves are consumers: wave w owns output rows iblk*32.. and channels pblk*32.. of every chunk and N/64
// of the 32x32 blocks of H; they run the MFMAs, gate, combine and store.  The last four waves are producers: one
// chunk ahead they compute Delta and the cumulative decay, build the masked decayed score operand, run conv + SiLU,
// and stage the C / B^T tiles, with the global loads of the chunk after that already in flight.  One LDS barrier per
// chunk.  (The producers' per-head work does not shrink with the head width, so their count does not either.)
// Block: 4*P + 256*PG threads.
// PG = 2 splits the producers into two groups of four waves: one builds the score operand and stages the tiles, the
// other runs conv + SiLU (both run the short scan for themselves).  A producer wave's chain of dependent stages per
// chunk is then about half as long, which is what sets the chunk period of long calls; the CU holds twelve waves.
// PARTS compiles the time parts in (chunk range and entry state per blockIdx.y); without it the kernel walks every
// chunk of its item and carries none of that bookkeeping through its loops.
// DUO (single-chunk calls only): both directions of a (batch, head) item in one workgroup, see ssd_duo_kernel.
// kDuoFirst is the direction that would park its result in global memory: it leaves it in LDS, one row per token.
// kDuoSecond is the direction that would read the parked result back: it takes it from `parked`, which its caller
// filled from LDS (register r: token i0 + row_k(r) of the thread's channel).
enum { kDuoNone = 0, kDuoFirst = 1, kDuoSecond = 2 };

// Where the first direction of a pair leaves its [kQ][P] fp32 result for the second: over the state operand copy
// when that is large enough (the first direction starts from a zero state and never reads it), else behind the
// scan tables.
template <int N, int P>
struct SsdDuoLds {
    using Lds = SsdLds<N, P, true>;
    static constexpr size_t kParkBytes = (size_t)kQ * P * sizeof(float);
    static constexpr bool kParkOverState = (size_t)Lds::kHT * sizeof(__bf16) >= kParkBytes;
    static constexpr size_t bytes() { return Lds::bytes() + (kParkOverState ? 0 : kParkBytes); }
};

template <int N, int P, bool SINGLE, int PG, bool PARTS, int DUO>
__device__ __forceinline__ void ssd_walk(const SsdArgs& a_in, float (&parked)[16])
{
    static_assert(PG == 1 || (PG == 2 && !SINGLE), "one or two producer groups; the single-chunk form keeps one");
    static_assert(!PARTS || (!SINGLE && PG == 1), "time parts come with one producer group and more than one chunk");
    static_assert(DUO == kDuoNone || SINGLE, "both directions in one workgroup: single-chunk calls only");
    using Lds = SsdLds<N, P, SINGLE>;
    SsdArgs a = a_in;
    if (SINGLE) a.nchunk = 1;   // known at compile time: the chunk pipeline below folds away
    constexpr int kPB = P / 32;       // channel blocks
    constexpr int kNB = N / 32;       // state blocks
    constexpr int kHB = kNB / 2;      // state blocks owned per consumer wave
    constexpr int kConsThreads = 4 * P;   // one consumer wave per 32 x 32 block of a chunk's output
    constexpr int kProdThreads = 256;
    constexpr int kRowC = Lds::kRowC, kRowT = Lds::kRowT;
    constexpr int kCopy = kQ * N / 8 / kProdThreads;   // 16-byte pieces of each tile per producer thread
    constexpr int kHS = 2 * 3 * 2 * 64 / kProdThreads;   // half operand slots (4 values) of the lower-triangular score blocks per producer thread
    using T = unsigned short;
    extern __shared__ __attribute__((aligned(16))) unsigned char ssd_lds[];
    __bf16* const tiles = reinterpret_cast<__bf16*>(ssd_lds);
    __bf16* const sHT = tiles + Lds::kBufs * Lds::kTileElems;
    float* const scal = reinterpret_cast<float*>(sHT + Lds::kBufs * Lds::kHT);   // [kBufs][kQ]: exp(l_i), decay from the chunk start
    float* const park = SsdDuoLds<N, P>::kParkOverState ? reinterpret_cast<float*>(sHT)
                                                        : scal + (Lds::kBufs + 3 * Lds::kScanTables) * kQ;   // DUO only
    auto sC = [&](int buf) { return tiles + buf * Lds::kTileElems; };
    auto sBT = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC; };
    auto sXc = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT; };
    auto sXw = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT + Lds::kX; };
    auto sM = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT + 2 * Lds::kX; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= kConsThreads / 64;
    // Workgroups go to the 8 XCDs round-robin by linear id and each XCD has its own L2.  All heads of a batch element
    // read the same C / B^T / score tiles, so the (batch, head) items are dealt out such that an XCD receives a
    // contiguous, batch-major run of them and fetches each tile from HBM once instead of once per XCD.
    int head = blockIdx.x, b = blockIdx.z;
    {
        const unsigned total = gridDim.x * gridDim.z, id = blockIdx.x + gridDim.x * blockIdx.z;
        if (total % 8 == 0) {
            const unsigned item = (id % 8) * (total / 8) + id / 8;
            head = (int)(item % gridDim.x);
            b = (int)(item / gridDim.x);
        }
    }
    const int grp = head / a.HG;
    const int ch0 = head * P;
    const size_t Lpad = (size_t)a.nchunk * kQ;
    // this workgroup's chunks [c_first, c_stop) and the states it starts from / leaves
    constexpr bool in_parts = PARTS;
    const int time_part = in_parts ? (int)blockIdx.y : 0;   // (`part` names the parked partial in the consumers)
    const int c_first = in_parts ? time_part * a.part_chunks : 0;
    const int c_stop = in_parts ? min(a.nchunk, c_first + a.part_chunks) : a.nchunk;
    const size_t part_elems = (size_t)gridDim.z * a.Dn * N;
    const float* const state_in = in_parts ? a.part_state + (size_t)time_part * a.part_subs * part_elems : a.h_in;
    float* const state_out = (time_part == (in_parts ? a.parts : 1) - 1) ? a.h_out : nullptr;
    const int last = a.L - 1;
    auto token_of = [&](int tau) { return a.dir > 0 ? tau : last - tau; };   // scan position -> token index

    if (producer) {
        // ------------------------------------------------------------------ producers
        constexpr int kCP = P / 2;                 // channel pairs of the head
        constexpr int kPos = kQ * kCP / kProdThreads;   // chunk positions per thread in the conv role (8 or 4)
        const int ptid = (tid - kConsThreads) % kProdThreads;    // index within the wave's group
        const int pwave = (wave - kConsThreads / 64) % 4;
        const int group = (wave - kConsThreads / 64) / 4;
        const bool do_score = PG == 1 || group == 0, do_conv = PG == 1 || group == 1;
        const int cp = ptid % kCP, tg = ptid / kCP;   // conv role: channels 2cp, 2cp+1; positions kPos*tg .. of each chunk
        // wave-private, written and read by this wave only (SINGLE: one copy, every wave writes the same values)
        float* const pw_l2 = scal + Lds::kBufs * kQ + (SINGLE ? 0 : pwave) * 3 * kQ;
        float* const pw_dl = pw_l2 + kQ;
        float* const pw_wgt = pw_dl + kQ;
        const float a2 = a.A[head] * kLog2e;
        const float dtb = (a.dt_softplus && a.dt_bias) ? a.dt_bias[head] : 0.0f;
        float w4[2][4], cbias[2];
#pragma unroll
        for (int h2 = 0; h2 < 2; h2++) {
#pragma unroll
            for (int i = 0; i < 4; i++)
                w4[h2][3 - i] = i < a.K ? a.conv_w[(size_t)(ch0 + 2 * cp + h2) * a.K + (a.K - 1 - i)] : 0.0f;
            cbias[h2] = a.conv_b ? a.conv_b[ch0 + 2 * cp + h2] : 0.0f;
        }
        const T* xb = (const T*)a.x.p + (size_t)b * a.x.sb + ch0 + 2 * cp;
        const T* dtp = (const T*)a.dt.p + (size_t)b * a.dt.sb + head;
        const long long xstep = a.dir * a.x.st;
        // this thread's 16-byte pieces of the C and B^T tiles: offsets inside a chunk (global) and inside the LDS tiles
        unsigned c_src[kCopy], b_src[kCopy], c_dst[kCopy], b_dst[kCopy];
#pragma unroll
        for (int i = 0; i < kCopy; i++) {
            const int idx = i * kProdThreads + ptid;
            c_src[i] = (unsigned)(idx / (N / 8)) * a.G * N + (idx % (N / 8)) * 8;
            b_src[i] = (idx / (kQ / 8)) * kQ + (idx % (kQ / 8)) * 8;
            c_dst[i] = (idx / (N / 8)) * kRowC + (idx % (N / 8)) * 8;
            b_dst[i] = (idx / (kQ / 8)) * kRowT + (idx % (kQ / 8)) * 8;
        }

        unsigned xraw[kPos + 3];   // channel pair at positions kPos*tg - 3 .. kPos*tg + kPos - 1
        T dtraw;
        bf16x8 ctile[kCopy], btile[kCopy];
        float4 gt[kHS];
        // Score operand half-slot hs = m*kProdThreads + ptid: slot hs/2 is block pair (iblk, jblk) = (0,0), (1,0), (1,1)
        // for hs / 256, k-block (hs / 128) % 2, operand lane (hs / 2) % 64; the half hs % 2 holds column
        // i = iblk*32 + lane%32 of rows j = jblk*32 + 16*kb + 8*(hs%2) + 4*(lane/32) + 0..3 (the accumulator-register
        // order, see the header comment).
        auto edge_chunk = [&](int c) { return c == 0 || c * kQ + kQ - 1 > last; };
        // The global loads of a chunk, one group per stage of `finish` (clamped positions: every address is valid).
        auto issue_dt = [&](int c) { dtraw = dtp[(long long)token_of(min(c * kQ + lane, last)) * a.dt.st]; };
        auto issue_score = [&](int c) {
            const float4* sc = reinterpret_cast<const float4*>(a.score_op + (((size_t)b * a.nchunk + c) * a.G + grp) * kScoreOp);
#pragma unroll
            for (int m = 0; m < kHS; m++) gt[m] = sc[m * kProdThreads + ptid];
        };
        auto issue_x = [&](int c) {
            const int tau0 = c * kQ + kPos * tg - 3;
            if (!edge_chunk(c)) {
                const T* xp = xb + (long long)token_of(tau0) * a.x.st;
#pragma unroll
                for (int q = 0; q < kPos + 3; q++) xraw[q] = *reinterpret_cast<const unsigned*>(xp + q * xstep);
            } else {
#pragma unroll
                for (int q = 0; q < kPos + 3; q++)
                    xraw[q] = *reinterpret_cast<const unsigned*>(xb + (long long)token_of(min(max(tau0 + q, 0), last)) * a.x.st);
            }
        };
        auto issue_tiles = [&](int c) {
            const __bf16* csrc = a.c_rows + (((size_t)b * Lpad + (size_t)c * kQ) * a.G + grp) * N;
            const __bf16* bsrc = a.b_t + ((((size_t)b * a.nchunk + c) * a.G + grp) * N) * kQ;
#pragma unroll
            for (int i = 0; i < kCopy; i++) {
                ctile[i] = *reinterpret_cast<const bf16x8*>(csrc + c_src[i]);
                btile[i] = *reinterpret_cast<const bf16x8*>(bsrc + b_src[i]);
            }
        };
        // Turn the data requested for chunk c into its tiles in buffer buf.  Each stage, once it has taken its inputs
        // out of the load registers, requests the same data of chunk cn (the chunk this wave handles next), so every
        // load has a whole chunk period to arrive.
        auto finish = [&](int c, int buf, int cn) {
            // Delta, inclusive cumulative log2-decay and end-of-chunk weight of position `lane` (every producer wave
            // computes them for itself; the first one publishes exp(l) for the consumers)
            float dl = IoBF16::cvt(dtraw);
            if (!SINGLE) issue_dt(cn);
            if (a.dt_softplus) dl = softplus(dl + dtb);
            if (c * kQ + lane > last) dl = 0.0f;
            const float l2 = wave_inclusive_sum(dl * a2);
            const float l2_end = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 63));
            // The decay exp(l_i - l_j) of a score element is separable, e_i f_j with e_i = exp(l_i - l_mid) and
            // f_j = exp(l_mid - l_j): two exponentials per position instead of one per element.  Both factors stay
            // well inside the fp32 range as long as the chunk's total decay does (2^-100 here); a chunk that decays
            // faster keeps the per-element form.
            const float l2_first = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 0));
            const float l2_mid = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), kQ / 2 - 1));
            const bool separable = l2_first - l2_end <= 100.0f;
            // (with two groups, wave i of each group shares slot i of the tables and writes only what its role reads)
            if (do_score) {
                if (separable) {
                    pw_l2[lane] = fast_exp2(l2 - l2_mid);          // e_i
                    pw_dl[lane] = fast_exp2(l2_mid - l2) * dl;     // f_j Delta_j
                } else {
                    pw_l2[lane] = l2;
                    pw_dl[lane] = dl;
                }
                if (pwave == 0) scal[buf * kQ + lane] = fast_exp2(l2);
            }
            if (do_conv) pw_wgt[lane] = fast_exp2(l2_end - l2) * dl;
            __builtin_amdgcn_wave_barrier();
            if (do_score) {
                // masked score operand: (B_j . C_i) exp(l_i - l_j) Delta_j for j <= i, else 0
                float sv[kHS][4];
#pragma unroll
                for (int m = 0; m < kHS; m++) { sv[m][0] = gt[m].x; sv[m][1] = gt[m].y; sv[m][2] = gt[m].z; sv[m][3] = gt[m].w; }
                asm volatile("" ::: "memory");   // the re-issue below must not move above the reads of gt
                if (!SINGLE) issue_score(cn);
#pragma unroll
                for (int m = 0; m < kHS; m++) {
                    const int hs = m * kProdThreads + ptid;
                    const int bp = hs / 256, kb = (hs / 128) % 2, sl = (hs / 2) % 64, hi = hs % 2;
                    const int iblk = bp > 0, jblk = bp > 1;
                    const int i = iblk * 32 + sl % 32;
                    const int jb = jblk * 32 + 16 * kb + 8 * hi + 4 * (sl / 32);
                    const bool diagonal = iblk == jblk;    // only the diagonal blocks hold elements with j > i
                    const float l2i = pw_l2[i];
                    const float4 da = *reinterpret_cast<const float4*>(&pw_dl[jb]);
                    const float dj[4] = {da.x, da.y, da.z, da.w};
                    bf16x4 v;
                    if (separable) {
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            const float val = sv[m][e] * l2i * dj[e];
                            v[e] = (__bf16)((diagonal && jb + e > i) ? 0.0f : val);
                        }
                    } else {
                        const float4 la = *reinterpret_cast<const float4*>(&pw_l2[jb]);
                        const float lj[4] = {la.x, la.y, la.z, la.w};
#pragma unroll
                        for (int e = 0; e < 4; e++) {
                            const float val = sv[m][e] * fast_exp2(l2i - lj[e]) * dj[e];
                            v[e] = (__bf16)((diagonal && jb + e > i) ? 0.0f : val);
                        }
                    }
                    *reinterpret_cast<bf16x4*>(&sM(buf)[(((iblk * 2 + jblk) * 2 + kb) * 64 + sl) * 8 + 4 * hi]) = v;
                }
            }
            if (do_conv) {
                // conv + SiLU of two channels at kPos positions
                float xr[2][kPos + 3];
#pragma unroll
                for (int q = 0; q < kPos + 3; q++) {
                    xr[0][q] = __uint_as_float(xraw[q] << 16);
                    xr[1][q] = __uint_as_float(xraw[q] & 0xffff0000u);
                }
                asm volatile("" ::: "memory");
                if (!SINGLE) issue_x(cn);
                if (edge_chunk(c)) {
#pragma unroll
                    for (int q = 0; q < kPos + 3; q++) {
                        const int tau = c * kQ + kPos * tg + q - 3;
                        if (tau < 0 || tau > last) xr[0][q] = xr[1][q] = 0.0f;
                    }
                    if (c == 0 && a.dir > 0 && a.tail_in && tg == 0 && a.K > 1) {
                        // requested together from clamped rows (a tap beyond the conv width has a zero weight)
                        T cached[3][2];
#pragma unroll
                        for (int q = 0; q < 3; q++) {   // 3 - q tokens before the block
                            const T* tp = (const T*)a.tail_in + ((size_t)b * (a.K - 1) + max(a.K - 1 - (3 - q), 0)) * a.tail_ch + ch0 + 2 * cp;
                            cached[q][0] = tp[0];
                            cached[q][1] = tp[1];
                        }
#pragma unroll
                        for (int q = 0; q < 3; q++) {
                            if (3 - q <= a.K - 1) {
                                xr[0][q] = IoBF16::cvt(cached[q][0]);
                                xr[1][q] = IoBF16::cvt(cached[q][1]);
                            }
                        }
                    }
                }
                float wq[kPos];
#pragma unroll
                for (int q = 0; q < kPos; q += 4) {
                    const float4 w = *reinterpret_cast<const float4*>(&pw_wgt[kPos * tg + q]);
                    wq[q] = w.x; wq[q + 1] = w.y; wq[q + 2] = w.z; wq[q + 3] = w.w;
                }
#pragma unroll
                for (int h2 = 0; h2 < 2; h2++) {
                    typedef __attribute__((__vector_size__(kPos * sizeof(__bf16)))) __bf16 bf16run;
                    bf16run vx, vw;
#pragma unroll
                    for (int q = 0; q < kPos; q++) {
                        float pre = cbias[h2];
                        pre = fmaf(w4[h2][0], xr[h2][q], pre);
                        pre = fmaf(w4[h2][1], xr[h2][q + 1], pre);
                        pre = fmaf(w4[h2][2], xr[h2][q + 2], pre);
                        pre = fmaf(w4[h2][3], xr[h2][q + 3], pre);
                        const float xc = silu(pre);
                        vx[q] = (__bf16)xc;
                        vw[q] = (__bf16)(xc * wq[q]);
                    }
                    *reinterpret_cast<bf16run*>(&sXc(buf)[(2 * cp + h2) * kRowT + kPos * tg]) = vx;
                    *reinterpret_cast<bf16run*>(&sXw(buf)[(2 * cp + h2) * kRowT + kPos * tg]) = vw;
                }
            }
            if (do_score) {
#pragma unroll
                for (int i = 0; i < kCopy; i++) {
                    *reinterpret_cast<bf16x8*>(&sC(buf)[c_dst[i]]) = ctile[i];
                    *reinterpret_cast<bf16x8*>(&sBT(buf)[b_dst[i]]) = btile[i];
                }
                asm volatile("" ::: "memory");
                if (!SINGLE) issue_tiles(cn);
            }
            __builtin_amdgcn_wave_barrier();   // the next chunk's scan results overwrite pw_* only after these reads
        };
        issue_dt(c_first);
        if (do_score) {
            issue_score(c_first);
            issue_tiles(c_first);
        }
        if (do_conv) issue_x(c_first);
        finish(c_first, 0, min(c_first + 1, c_stop - 1));
        lds_barrier();
        for (int c = c_first; c < c_stop; c++) {
            if (c + 1 < c_stop) finish(c + 1, (c + 1 - c_first) & 1, min(c + 2, c_stop - 1));
            lds_barrier();
        }
        return;
    }

    // ---------------------------------------------------------------------- consumers
    // The output mode is fixed per launch; the walk is compiled once per mode so that the per-chunk code has no
    // mode branches (gfx9 counts loads and stores on one counter: a load awaited while a store is in flight costs
    // the store's full round trip, so every chunk first consumes its prefetched gate data, then stores).
    auto walk = [&](auto mode_c) {
        constexpr int kMode = decltype(mode_c)::value;
        constexpr bool need_z = kMode != kSsdPartialRaw;
        constexpr bool adds_parked = kMode == kSsdFinalAdd || kMode == kSsdFinalAddRaw;
        constexpr bool need_p = adds_parked && DUO != kDuoSecond;   // read back from global memory
        constexpr bool parks = kMode == kSsdPartialRaw || kMode == kSsdPartial;
        const int iblk = wave / kPB, pblk = wave % kPB;
        const int cl = lane & 31, half = lane >> 5;
        const int po = pblk * 32 + cl;             // this lane's channel within the head
        const int icol = iblk * 32 + cl;           // this lane's output row, as the score tile's column
        const int i0 = iblk * 32 + 4 * half;       // output row of accumulator register 0; register r: i0 + row_k(r)
        auto row_k = [](int r) { return 8 * (r / 4) + (r % 4); };
        const float dval = a.D[a.d_per_head ? head : ch0 + po];
        const T* zb = (const T*)a.z.p + (size_t)b * a.z.sb + ch0 + po;
        float* const pbase = a.partial + (size_t)b * a.L * a.Dn + ch0 + po;
        T* const obase = (T*)a.out + (size_t)b * a.out_sb + a.out_ch_off + ch0 + po;
        // signed element steps from one scan position to the next
        const long long zstep = a.dir * a.z.st, pstep = (long long)a.dir * a.Dn, ostep = a.dir * a.out_st;

        f32x16 hacc[kHB];
#pragma unroll
        for (int hb = 0; hb < kHB; hb++) {
            const int nblk = iblk * kHB + hb;
#pragma unroll
            for (int r = 0; r < 16; r++) hacc[hb][r] = 0.0f;
            if (state_in) {   // registers 4q .. 4q+3 hold four adjacent states: 16-byte pieces (the host checks alignment)
                const float* hrow = state_in + ((size_t)b * a.Dn + ch0 + po) * N + nblk * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float4 v = *reinterpret_cast<const float4*>(hrow + 8 * q);
                    hacc[hb][4 * q] = v.x; hacc[hb][4 * q + 1] = v.y; hacc[hb][4 * q + 2] = v.z; hacc[hb][4 * q + 3] = v.w;
                }
            }
        }
        auto publish_state = [&](int which) {
#pragma unroll
            for (int hb = 0; hb < kHB; hb++) {
                const int nblk = iblk * kHB + hb;
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    bf16x8 v;
#pragma unroll
                    for (int e = 0; e < 8; e++) v[e] = (__bf16)hacc[hb][8 * kb + e];
                    *reinterpret_cast<bf16x8*>(&sHT[which * Lds::kHT + (((nblk * kPB + pblk) * 2 + kb) * 64 + lane) * 8]) = v;
                }
            }
        };
        // gate and parked partial of one chunk, requested a whole chunk before they are used.  A chunk that ends
        // inside the sequence addresses its rows as one base plus constant multiples of the step; the ragged last
        // chunk clamps every position instead.
        T zraw[16];
        float part[16];
        if constexpr (DUO == kDuoSecond && adds_parked) {
#pragma unroll
            for (int r = 0; r < 16; r++) part[r] = parked[r];
        }
        auto issue_gate = [&](int c) {
            const int tau0 = c * kQ + i0;
            if (c * kQ + kQ - 1 <= last) {
                const long long t0 = token_of(tau0);
                const T* zp = zb + t0 * a.z.st;
                const float* pp = pbase + t0 * a.Dn;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    if constexpr (need_z) zraw[r] = zp[row_k(r) * zstep];
                    if constexpr (need_p) part[r] = pp[row_k(r) * pstep];
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const long long t = token_of(min(tau0 + row_k(r), last));
                    if constexpr (need_z) zraw[r] = zb[t * a.z.st];
                    if constexpr (need_p) part[r] = pbase[t * a.Dn];
                }
            }
        };
        publish_state(0);
        bool state_nonzero = state_in != nullptr;
        issue_gate(c_first);
        lds_barrier();

        for (int c = c_first; c < c_stop; c++) {
            const int buf = (c - c_first) & 1;
            const float* el = scal + buf * kQ;
            const __bf16* xc_t = sXc(buf);
            // ---- intra-chunk product with the masked, decayed score operand the producers prepared
            f32x16 y1 = {0}, y2 = {0};
#pragma unroll
            for (int jblk = 0; jblk < 2; jblk++) {
                if (jblk > iblk) break;
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    const bf16x8 am = *reinterpret_cast<const bf16x8*>(&sM(buf)[(((iblk * 2 + jblk) * 2 + kb) * 64 + lane) * 8]);
                    bf16x8 bx;
#pragma unroll
                    for (int jj = 0; jj < 2; jj++) {
                        const bf16x4 v = *reinterpret_cast<const bf16x4*>(&xc_t[po * kRowT + jblk * 32 + 16 * kb + 8 * jj + 4 * half]);
#pragma unroll
                        for (int e = 0; e < 4; e++) bx[4 * jj + e] = v[e];
                    }
                    y1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bx, y1, 0, 0, 0);
                }
            }
            // ---- inter-chunk product with the state entering the chunk
            if (state_nonzero) {
                const __bf16* c_t = sC(buf);
                const __bf16* h_t = sHT + buf * Lds::kHT;
#pragma unroll
                for (int nblk = 0; nblk < kNB; nblk++) {
#pragma unroll
                    for (int kb = 0; kb < 2; kb++) {
                        bf16x8 ac;
#pragma unroll
                        for (int jj = 0; jj < 2; jj++) {
                            const bf16x4 v = *reinterpret_cast<const bf16x4*>(&c_t[icol * kRowC + nblk * 32 + 16 * kb + 8 * jj + 4 * half]);
#pragma unroll
                            for (int e = 0; e < 4; e++) ac[4 * jj + e] = v[e];
                        }
                        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(&h_t[(((nblk * kPB + pblk) * 2 + kb) * 64 + lane) * 8]);
                        y2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac, bh, y2, 0, 0, 0);
                    }
                }
            }
            // ---- state update of the blocks this wave owns (the state after the last chunk matters only if it is
            // committed)
            const bool state_needed = c + 1 < c_stop || state_out != nullptr;
            if (state_needed) {
                const __bf16* b_t = sBT(buf);
                const __bf16* xw_t = sXw(buf);
                const float decay_q = el[kQ - 1];
#pragma unroll
                for (int hb = 0; hb < kHB; hb++) {
                    const int nblk = iblk * kHB + hb;
#pragma unroll
                    for (int r = 0; r < 16; r++) hacc[hb][r] *= decay_q;
#pragma unroll
                    for (int kb = 0; kb < 4; kb++) {
                        const bf16x8 ab = *reinterpret_cast<const bf16x8*>(&b_t[(nblk * 32 + cl) * kRowT + 16 * kb + 8 * half]);
                        const bf16x8 bw = *reinterpret_cast<const bf16x8*>(&xw_t[po * kRowT + 16 * kb + 8 * half]);
                        hacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bw, hacc[hb], 0, 0, 0);
                    }
                }
            }
            // ---- epilogue: inter-chunk term, skip term, gate, combine; all 16 results first, then the stores
            {
                float res[16];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float4 e4 = *reinterpret_cast<const float4*>(&el[i0 + 8 * q]);
                    const bf16x4 x4 = *reinterpret_cast<const bf16x4*>(&xc_t[po * kRowT + i0 + 8 * q]);
                    const float ev[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const int r = 4 * q + e;
                        const float y = y1[r] + ev[e] * y2[r] + dval * (float)x4[e];
                        if constexpr (!need_z) res[r] = y;
                        else {
                            const float zg = silu(IoBF16::cvt(zraw[r]));
                            res[r] = kMode == kSsdFinalAddRaw ? (y + part[r]) * zg : adds_parked ? y * zg + part[r] : y * zg;
                        }
                    }
                }
                {
                    const int tau0 = c * kQ + i0;
                    if (c * kQ + kQ - 1 <= last) {
                        const long long t0 = token_of(tau0);
                        float* pp = pbase + t0 * a.Dn;
                        T* op = obase + t0 * a.out_st;
#pragma unroll
                        for (int r = 0; r < 16; r++) {
                            if constexpr (parks && DUO == kDuoFirst) park[((int)t0 + row_k(r) * a.dir) * P + po] = res[r];
                            else if constexpr (parks) pp[row_k(r) * pstep] = res[r];
                            else IoBF16::st(op + row_k(r) * ostep, res[r]);
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; r++) {
                            const int tau = tau0 + row_k(r);
                            if (tau <= last) {
                                const long long t = token_of(tau);
                                if constexpr (parks && DUO == kDuoFirst) park[(int)t * P + po] = res[r];
                                else if constexpr (parks) pbase[t * a.Dn] = res[r];
                                else IoBF16::st(obase + t * a.out_st, res[r]);
                            }
                        }
                    }
                }
            }
            if (c + 1 < c_stop) {
                issue_gate(c + 1);
                publish_state(buf ^ 1);
            }
            state_nonzero = true;
            lds_barrier();
        }
        if (state_out) {
#pragma unroll
            for (int hb = 0; hb < kHB; hb++) {
                const int nblk = iblk * kHB + hb;
                float* hrow = state_out + ((size_t)b * a.Dn + ch0 + po) * N + nblk * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    *reinterpret_cast<float4*>(hrow + 8 * q) =
                        make_float4(hacc[hb][4 * q], hacc[hb][4 * q + 1], hacc[hb][4 * q + 2], hacc[hb][4 * q + 3]);
            }
        }
    };
    if constexpr (DUO == kDuoFirst) {   // the direction that parks (or stores its own half of a two-part output)
        switch (a.mode) {
            case kSsdFinalOnly: walk(std::integral_constant<int, kSsdFinalOnly>{}); break;
            case kSsdPartial: walk(std::integral_constant<int, kSsdPartial>{}); break;
            default: walk(std::integral_constant<int, kSsdPartialRaw>{}); break;
        }
    } else if constexpr (DUO == kDuoSecond) {
        switch (a.mode) {
            case kSsdFinalOnly: walk(std::integral_constant<int, kSsdFinalOnly>{}); break;
            case kSsdFinalAdd: walk(std::integral_constant<int, kSsdFinalAdd>{}); break;
            default: walk(std::integral_constant<int, kSsdFinalAddRaw>{}); break;
        }
    } else {
        switch (a.mode) {
            case kSsdFinalOnly: walk(std::integral_constant<int, kSsdFinalOnly>{}); break;
            case kSsdPartial: walk(std::integral_constant<int, kSsdPartial>{}); break;
            case kSsdPartialRaw: walk(std::integral_constant<int, kSsdPartialRaw>{}); break;
            case kSsdFinalAdd: walk(std::integral_constant<int, kSsdFinalAdd>{}); break;
            default: walk(std::integral_constant<int, kSsdFinalAddRaw>{}); break;
        }
    }
}

template <int N, int P, bool SINGLE = false, int PG = 1, bool PARTS = false>
__global__ __launch_bounds__(4 * P + 256 * PG, SINGLE ? 4 : 1) void ssd_kernel(const SsdArgs a)
{
    float none[16];
    ssd_walk<N, P, SINGLE, PG, PARTS, kDuoNone>(a, none);
}

// Single-chunk calls (block-diffusion steps), both directions of a (batch, head) item in one workgroup: the reverse
// direction runs first and leaves its result in LDS instead of parking it in global memory, the forward direction
// picks it up, so the call is one scan launch instead of two, x's rows are fetched from HBM once and the partial
// never leaves the chip.  grid (H, 1, batch), block 4*P + 256, dynamic LDS SsdDuoLds<N, P>::bytes().  Between the
// directions every consumer thread takes the 16 parked values of its (token, channel) places into registers, then a
// barrier lets the forward direction overwrite the tiles and the state operand copy.
template <int N, int P>
__global__ __launch_bounds__(4 * P + 256, 4) void ssd_duo_kernel(const SsdStatePair both)
{
    using Lds = SsdLds<N, P, true>;
    float parked[16];
#pragma unroll
    for (int r = 0; r < 16; r++) parked[r] = 0.0f;
    ssd_walk<N, P, true, 1, false, kDuoFirst>(both.dir[1], parked);
    const int tid = threadIdx.x;
    if (tid < 4 * P && both.dir[1].mode != kSsdFinalOnly) {   // consumer waves, same places as in ssd_walk
        extern __shared__ __attribute__((aligned(16))) unsigned char ssd_lds[];
        __bf16* const sHT = reinterpret_cast<__bf16*>(ssd_lds) + Lds::kTileElems;
        const float* const park = SsdDuoLds<N, P>::kParkOverState
                                      ? reinterpret_cast<const float*>(sHT)
                                      : reinterpret_cast<const float*>(sHT + Lds::kHT) + (1 + 3) * kQ;
        const int wave = tid >> 6, lane = tid & 63;
        const int iblk = wave / (P / 32), pblk = wave % (P / 32);
        const int po = pblk * 32 + (lane & 31), i0 = iblk * 32 + 4 * (lane >> 5);
        const int last = both.dir[0].L - 1;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int t = i0 + 8 * (r / 4) + (r % 4);
            parked[r] = t <= last ? park[t * P + po] : 0.0f;
        }
    }
    lds_barrier();
    ssd_walk<N, P, true, 1, false, kDuoSecond>(both.dir[0], parked);
}

}  // namespace bm
