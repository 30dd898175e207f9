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
// Lane layouts of the 32x32x16 MFMA (checked on hardware): operand A lane l holds row l%32, k = 8*(l/32)..+7;
// operand B lane l holds column l%32, same k; accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4,
// column l%32.  A contraction index may be enumerated in any order as long as both operands agree, which lets an
// accumulator tile be fed back as an operand without a transpose: registers 8*kb..8*kb+7 of a lane are the 8
// k-slots of k-block kb, i.e. k = 16*kb + 8*jj + 4*(l/32) + e for slot 4*jj + e.
#pragma once
#include "kernels.h"

namespace bm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kQ = 64;     // chunk length
constexpr int kPadK = 8;   // bf16 elements of row padding in LDS tiles (keeps 16-byte alignment, spreads banks)

struct SsdPrepArgs {
    const float* bc;   // fp32 B|C rows [batch][L][G][2N] in token order (from prep_bc_kernel)
    __bf16* c_rows;    // [batch][Lpad][G][N], scan order
    __bf16* b_t;       // [batch][nchunk][G][N][64], scan order inside the chunk
    float* score_t;    // [batch][nchunk][G][64 j][64 i] = B_j . C_i
    int L, G, dir;     // dir +1: scan position tau is token tau; -1: token L-1-tau
};

template <int N>
constexpr size_t ssd_prep_lds_bytes() { return 2 * (size_t)kQ * (N + 1) * sizeof(float); }

// grid (nchunk, G, batch), block 256, dynamic LDS ssd_prep_lds_bytes<N>()
template <int N>
__global__ __launch_bounds__(256) void ssd_prep_kernel(const SsdPrepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ssd_prep_lds[];
    float(*sB)[N + 1] = reinterpret_cast<float(*)[N + 1]>(ssd_prep_lds);
    float(*sC)[N + 1] = sB + kQ;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int nchunk = gridDim.x;
    for (int idx = tid; idx < kQ * 2 * N; idx += 256) {
        const int j = idx / (2 * N), col = idx % (2 * N);
        const int tau = c * kQ + j;
        float v = 0.0f;
        if (tau < a.L) {
            const int t = a.dir > 0 ? tau : a.L - 1 - tau;
            v = a.bc[(((size_t)b * a.L + t) * a.G + g) * (2 * N) + col];
        }
        if (col < N) sB[j][col] = v;
        else sC[j][col - N] = v;
    }
    __syncthreads();
    const size_t Lpad = (size_t)nchunk * kQ;
    for (int idx = tid; idx < kQ * N; idx += 256) {
        const int j = idx / N, n = idx % N;
        a.c_rows[(((size_t)b * Lpad + c * kQ + j) * a.G + g) * N + n] = (__bf16)sC[j][n];
        const int n2 = idx / kQ, j2 = idx % kQ;
        a.b_t[((((size_t)b * nchunk + c) * a.G + g) * N + n2) * kQ + j2] = (__bf16)sB[j2][n2];
    }
    // 4 x 4 outputs per thread
    const int tj = tid / 16, ti = tid % 16;
    float acc[4][4] = {};
    for (int n = 0; n < N; n++) {
        float bv[4], cv[4];
#pragma unroll
        for (int q = 0; q < 4; q++) { bv[q] = sB[4 * tj + q][n]; cv[q] = sC[4 * ti + q][n]; }
#pragma unroll
        for (int q = 0; q < 4; q++)
#pragma unroll
            for (int r = 0; r < 4; r++) acc[q][r] = fmaf(bv[q], cv[r], acc[q][r]);
    }
    float* dst = a.score_t + (((size_t)b * nchunk + c) * a.G + g) * (kQ * kQ);
#pragma unroll
    for (int q = 0; q < 4; q++)
        *reinterpret_cast<float4*>(dst + (4 * tj + q) * kQ + 4 * ti) = make_float4(acc[q][0], acc[q][1], acc[q][2], acc[q][3]);
}

enum { kSsdFinalOnly = 0, kSsdPartial = 1, kSsdPartialRaw = 2, kSsdFinalAdd = 3, kSsdFinalAddRaw = 4 };

struct SsdArgs {
    TensorArg x, z, dt;
    const float *conv_w, *conv_b, *A, *D, *dt_bias;
    const __bf16* c_rows;
    const __bf16* b_t;
    const float* score_t;
    void* out;
    long long out_sb, out_st;
    float* partial;       // [batch][L][Dn] fp32
    const float* h_in;    // [batch][Dn][N] or null
    float* h_out;         // or null
    const void* tail_in;  // bf16 [batch][K-1][tail_ch] or null (causal direction only)
    int L, Dn, H, HG, G, K, tail_ch, nchunk;
    int dir, mode, out_ch_off, dt_softplus, d_per_head;
};

template <int N, int P>
constexpr size_t ssd_lds_bytes()
{
    return ((size_t)kQ * (N + kPadK) + (size_t)N * (kQ + kPadK) + 2 * (size_t)P * (kQ + kPadK) + (size_t)(N / 32) * (P / 32) * 2 * 64 * 8) *
               sizeof(__bf16) + 3 * kQ * sizeof(float);
}

// grid (H, 1, batch), block 4*P, dynamic LDS ssd_lds_bytes<N, P>(): wave w owns output rows iblk*32.. and channels pblk*32.. of every chunk,
// and N/64 of the 32x32 blocks of H.
template <int N, int P>
__global__ __launch_bounds__(4 * P) void ssd_kernel(const SsdArgs a)
{
    constexpr int kPB = P / 32;       // channel blocks
    constexpr int kNB = N / 32;       // state blocks
    constexpr int kHB = kNB / 2;      // state blocks owned per wave
    constexpr int kThreads = 4 * P;
    constexpr int kRowC = N + kPadK, kRowT = kQ + kPadK;
    using T = unsigned short;
    extern __shared__ __attribute__((aligned(16))) unsigned char ssd_lds[];
    __bf16* sC = reinterpret_cast<__bf16*>(ssd_lds);   // [kQ][kRowC]   C rows of the chunk
    __bf16* sBT = sC + kQ * kRowC;                      // [N][kRowT]    B transposed
    __bf16* sXc = sBT + N * kRowT;                      // [P][kRowT]    conv + SiLU output, transposed
    __bf16* sXw = sXc + P * kRowT;                      // [P][kRowT]    same, scaled by exp(l_Q - l_j) Delta_j
    __bf16* sHT = sXw + P * kRowT;                      // [kNB][kPB][2][64][8]  state as an MFMA operand
    float* sL2 = reinterpret_cast<float*>(sHT + kNB * kPB * 2 * 64 * 8);
    float* sDl = sL2 + kQ;
    float* sW = sDl + kQ;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int iblk = wave / kPB, pblk = wave % kPB;
    const int cl = lane & 31, half = lane >> 5;
    const int head = blockIdx.x, b = blockIdx.z;
    const int grp = head / a.HG;
    const int ch0 = head * P;
    const float a2 = a.A[head] * kLog2e;
    const float dtb = (a.dt_softplus && a.dt_bias) ? a.dt_bias[head] : 0.0f;

    // conv role: channel pc, tokens 16*tg .. 16*tg+15 of each chunk
    const int pc = tid % P, tg = tid / P;
    float w4[4];
#pragma unroll
    for (int i = 0; i < 4; i++) w4[3 - i] = i < a.K ? a.conv_w[(size_t)(ch0 + pc) * a.K + (a.K - 1 - i)] : 0.0f;
    const float cbias = a.conv_b ? a.conv_b[ch0 + pc] : 0.0f;
    // output role: channel po
    const int po = pblk * 32 + cl;
    const float dval = a.D[a.d_per_head ? head : ch0 + po];

    // state blocks in accumulator layout
    f32x16 hacc[kHB];
#pragma unroll
    for (int hb = 0; hb < kHB; hb++) {
        const int nblk = iblk * kHB + hb;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const int n = nblk * 32 + 8 * (r / 4) + 4 * half + (r % 4);
            hacc[hb][r] = a.h_in ? a.h_in[((size_t)b * a.Dn + ch0 + po) * N + n] : 0.0f;
        }
    }
    auto publish_state = [&]() {
#pragma unroll
        for (int hb = 0; hb < kHB; hb++) {
            const int nblk = iblk * kHB + hb;
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                bf16x8 v;
#pragma unroll
                for (int e = 0; e < 8; e++) v[e] = (__bf16)hacc[hb][8 * kb + e];
                *reinterpret_cast<bf16x8*>(&sHT[(((nblk * kPB + pblk) * 2 + kb) * 64 + lane) * 8]) = v;
            }
        }
    };
    publish_state();
    bool state_nonzero = a.h_in != nullptr;

    const T* xb = (const T*)a.x.p + (size_t)b * a.x.sb + ch0;
    const T* zb = (const T*)a.z.p + (size_t)b * a.z.sb + ch0;
    const T* dtb_p = (const T*)a.dt.p + (size_t)b * a.dt.sb + head;
    const size_t Lpad = (size_t)a.nchunk * kQ;

    for (int c = 0; c < a.nchunk; c++) {
        // ---- A1: Delta, cumulative log-decay (base 2) and end-of-chunk weights, by wave 0
        if (wave == 0) {
            const int tau = c * kQ + lane;
            const int tc = min(tau, a.L - 1);
            float dl = IoBF16::ld(dtb_p + (long long)(a.dir > 0 ? tc : a.L - 1 - tc) * a.dt.st);
            if (a.dt_softplus) dl = softplus(dl + dtb);
            if (tau >= a.L) dl = 0.0f;
            float l2 = dl * a2;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float up = __shfl_up(l2, off, 64);
                if (lane >= off) l2 += up;
            }
            const float l2q = __shfl(l2, 63, 64);
            sL2[lane] = l2;
            sDl[lane] = dl;
            sW[lane] = fast_exp2(l2q - l2) * dl;
        }
        // x of this thread's 16 tokens plus the 3 before them in scan order: every load is issued unconditionally from
        // a clamped position (so the 19 requests overlap) and zeroed by a select when the position is outside [0, L)
        float xr[19];
#pragma unroll
        for (int q = 0; q < 19; q++) {
            const int tau = c * kQ + 16 * tg + q - 3;
            const int tc = min(max(tau, 0), a.L - 1);
            const int t = a.dir > 0 ? tc : a.L - 1 - tc;
            const float v = IoBF16::ld(xb + (long long)t * a.x.st + pc);
            xr[q] = (tau >= 0 && tau < a.L) ? v : 0.0f;
        }
        if (c == 0 && tg == 0 && a.dir > 0 && a.tail_in) {
#pragma unroll
            for (int q = 0; q < 3; q++) {
                const int tau = q - 3;
                if (tau + (a.K - 1) >= 0)
                    xr[q] = IoBF16::ld((const T*)a.tail_in + ((size_t)b * (a.K - 1) + (a.K - 1 + tau)) * a.tail_ch + ch0 + pc);
            }
        }
        // C rows and transposed B tile of this chunk into LDS, 16 bytes at a time
        {
            const __bf16* csrc = a.c_rows + (((size_t)b * Lpad + (size_t)c * kQ) * a.G + grp) * N;
            for (int idx = tid; idx < kQ * N / 8; idx += kThreads) {
                const int j = idx / (N / 8), col = (idx % (N / 8)) * 8;
                *reinterpret_cast<bf16x8*>(&sC[j * kRowC + col]) =
                    *reinterpret_cast<const bf16x8*>(csrc + (size_t)j * a.G * N + col);
            }
            const __bf16* bsrc = a.b_t + ((((size_t)b * a.nchunk + c) * a.G + grp) * N) * kQ;
            for (int idx = tid; idx < N * kQ / 8; idx += kThreads) {
                const int n = idx / (kQ / 8), col = (idx % (kQ / 8)) * 8;
                *reinterpret_cast<bf16x8*>(&sBT[n * kRowT + col]) = *reinterpret_cast<const bf16x8*>(bsrc + n * kQ + col);
            }
        }
        __syncthreads();
        // ---- A2: conv + SiLU, two bf16 copies transposed to [channel][position]
        {
            bf16x8 vx[2], vw[2];
#pragma unroll
            for (int q = 0; q < 16; q++) {
                float pre = cbias;
                pre = fmaf(w4[0], xr[q], pre);
                pre = fmaf(w4[1], xr[q + 1], pre);
                pre = fmaf(w4[2], xr[q + 2], pre);
                pre = fmaf(w4[3], xr[q + 3], pre);
                const float xc = silu(pre);
                vx[q / 8][q % 8] = (__bf16)xc;
                vw[q / 8][q % 8] = (__bf16)(xc * sW[16 * tg + q]);
            }
#pragma unroll
            for (int q = 0; q < 2; q++) {
                *reinterpret_cast<bf16x8*>(&sXc[pc * kRowT + 16 * tg + 8 * q]) = vx[q];
                *reinterpret_cast<bf16x8*>(&sXw[pc * kRowT + 16 * tg + 8 * q]) = vw[q];
            }
        }
        __syncthreads();
        // ---- B: outputs of this chunk
        f32x16 y1 = {0}, y2 = {0};
        const int icol = iblk * 32 + cl;  // this lane's output row as the score tile's column
        const float l2i = sL2[icol];
        for (int jblk = 0; jblk <= iblk; jblk++) {
            const float* sc = a.score_t + (((size_t)b * a.nchunk + c) * a.G + grp) * (kQ * kQ);
            float gt[16];
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int j = jblk * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                gt[r] = sc[j * kQ + icol];
            }
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                bf16x8 am, bx;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const int r = 8 * kb + e;
                    const int j = jblk * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                    float m = gt[r] * fast_exp2(l2i - sL2[j]) * sDl[j];
                    if (j > icol) m = 0.0f;
                    am[e] = (__bf16)m;
                }
#pragma unroll
                for (int jj = 0; jj < 2; jj++) {
                    const bf16x4 v = *reinterpret_cast<const bf16x4*>(&sXc[po * kRowT + jblk * 32 + 16 * kb + 8 * jj + 4 * half]);
#pragma unroll
                    for (int e = 0; e < 4; e++) bx[4 * jj + e] = v[e];
                }
                y1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bx, y1, 0, 0, 0);
            }
        }
        if (state_nonzero) {
#pragma unroll
            for (int nblk = 0; nblk < kNB; nblk++) {
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    bf16x8 ac;
#pragma unroll
                    for (int jj = 0; jj < 2; jj++) {
                        const bf16x4 v = *reinterpret_cast<const bf16x4*>(&sC[icol * kRowC + nblk * 32 + 16 * kb + 8 * jj + 4 * half]);
#pragma unroll
                        for (int e = 0; e < 4; e++) ac[4 * jj + e] = v[e];
                    }
                    const bf16x8 bh = *reinterpret_cast<const bf16x8*>(&sHT[(((nblk * kPB + pblk) * 2 + kb) * 64 + lane) * 8]);
                    y2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac, bh, y2, 0, 0, 0);
                }
            }
        }
        // ---- C: state update of the blocks this wave owns
        {
            const float decay_q = fast_exp2(sL2[kQ - 1]);
#pragma unroll
            for (int hb = 0; hb < kHB; hb++) {
                const int nblk = iblk * kHB + hb;
#pragma unroll
                for (int r = 0; r < 16; r++) hacc[hb][r] *= decay_q;
#pragma unroll
                for (int kb = 0; kb < 4; kb++) {
                    const bf16x8 ab = *reinterpret_cast<const bf16x8*>(&sBT[(nblk * 32 + cl) * kRowT + 16 * kb + 8 * half]);
                    const bf16x8 bw = *reinterpret_cast<const bf16x8*>(&sXw[po * kRowT + 16 * kb + 8 * half]);
                    hacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bw, hacc[hb], 0, 0, 0);
                }
            }
        }
        // ---- epilogue: inter-chunk term, skip term, gate, combine, store.  Gate and partial values of the 16 outputs are
        // requested together from clamped positions before any of them is used.
        {
            const bool need_z = a.mode != kSsdPartialRaw;
            const bool need_p = a.mode == kSsdFinalAdd || a.mode == kSsdFinalAddRaw;
            T zraw[16];
            float part[16];
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int tau = min(c * kQ + iblk * 32 + 8 * (r / 4) + 4 * half + (r % 4), a.L - 1);
                const int t = a.dir > 0 ? tau : a.L - 1 - tau;
                zraw[r] = need_z ? zb[(long long)t * a.z.st + po] : (T)0;
                part[r] = need_p ? a.partial[((size_t)b * a.L + t) * a.Dn + ch0 + po] : 0.0f;
            }
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int i = iblk * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                const int tau = c * kQ + i;
                const int t = a.dir > 0 ? tau : a.L - 1 - tau;
                const float y = y1[r] + fast_exp2(sL2[i]) * y2[r] + dval * (float)sXc[po * kRowT + i];
                float res;
                if (a.mode == kSsdPartialRaw) res = y;
                else {
                    const float zg = silu(IoBF16::cvt(zraw[r]));
                    res = a.mode == kSsdFinalAddRaw ? (y + part[r]) * zg : y * zg + part[r];
                }
                if (tau < a.L) {
                    if (a.mode == kSsdPartialRaw || a.mode == kSsdPartial)
                        a.partial[((size_t)b * a.L + t) * a.Dn + ch0 + po] = res;
                    else
                        IoBF16::st((T*)a.out + (size_t)b * a.out_sb + (long long)t * a.out_st + a.out_ch_off + ch0 + po, res);
                }
            }
        }
        __syncthreads();  // every wave is done with this chunk's tiles and with the published state
        publish_state();
        state_nonzero = true;
    }
    if (a.h_out) {
#pragma unroll
        for (int hb = 0; hb < kHB; hb++) {
            const int nblk = iblk * kHB + hb;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int n = nblk * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                a.h_out[((size_t)b * a.Dn + ch0 + po) * N + n] = hacc[hb][r];
            }
        }
    }
}

}  // namespace bm
