// The chunk walk of ssd_kernels.h for calls that fill the chip, as sixteen short instruction streams instead of eight.
//
// A wave issues at most one instruction every six to seven cycles whatever the instruction is, while a SIMD's vector
// ALU accepts a 64-lane instruction every four, so a workgroup is as fast as its longest per-chunk instruction stream,
// not as its total work.  ssd_kernel deals a chunk to four consumer and four producer waves; here the same work goes to
//   y waves   (P/16): the intra-chunk product, the inter-chunk product C H and the epilogue of a 32 x 32 output block;
//   h waves   (N/32): the state update of one row block of H (all channel blocks, so one B^T operand serves them all),
//                     its decay and the bf16 operand copy of the new state;
//   producers (8):    four build the masked, decayed score operand and stage the C / B^T tiles, four run conv + SiLU.
// Tiles, double buffering and the one barrier per chunk are those of ssd_kernel.  The epilogue addresses the rows of a
// chunk through raw buffer ranges (a constant lane offset per row group plus a scalar row offset: no vector address
// arithmetic), and the result one direction parks for the other crosses global memory as bf16: in the paper's
// precision (bf16 autocast, App. A) each direction's output is a bf16 tensor before the two are added (eq. 6).
//
// Multi-chunk calls without time parts only; z / out token strides up to 2^24 elements (the host checks).
#pragma once
#include "ssd_kernels.h"

namespace bm {

template <int N, int P>
struct SsdWide {
    static constexpr int kPB = P / 32, kNB = N / 32;
    static constexpr int kYWaves = 2 * kPB, kHWaves = kNB, kProdWaves = 8;
    static constexpr int kThreads = 64 * (kYWaves + kHWaves + kProdWaves);
};

template <int N, int P>
__global__ __launch_bounds__((SsdWide<N, P>::kThreads)) void ssd_wide_kernel(const SsdArgs a)
{
    using Lds = SsdLds<N, P, false>;
    using W = SsdWide<N, P>;
    constexpr int kPB = W::kPB, kNB = W::kNB;
    constexpr int kProdThreads = 256;
    constexpr int kRowC = Lds::kRowC, kRowT = Lds::kRowT;
    constexpr int kCopy = kQ * N / 8 / kProdThreads;
    constexpr int kHS = 2 * 3 * 2 * 64 / kProdThreads;
    using T = unsigned short;
    extern __shared__ __attribute__((aligned(16))) unsigned char ssd_lds[];
    __bf16* const tiles = reinterpret_cast<__bf16*>(ssd_lds);
    __bf16* const sHT = tiles + Lds::kBufs * Lds::kTileElems;
    float* const scal = reinterpret_cast<float*>(sHT + Lds::kBufs * Lds::kHT);
    auto sC = [&](int buf) { return tiles + buf * Lds::kTileElems; };
    auto sBT = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC; };
    auto sXc = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT; };
    auto sXw = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT + Lds::kX; };
    auto sM = [&](int buf) { return tiles + buf * Lds::kTileElems + Lds::kC + Lds::kBT + 2 * Lds::kX; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // (batch, head) items dealt to the XCDs batch-major, as in ssd_walk: the heads of a batch element share their tiles
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
    const int nchunk = a.nchunk;
    const int last = a.L - 1;
    auto token_of = [&](int tau) { return a.dir > 0 ? tau : last - tau; };
    const int cl = lane & 31, half = lane >> 5;

    if (wave >= W::kYWaves + W::kHWaves) {
        // ------------------------------------------------------------------ producers (two groups of four waves)
        constexpr int kCP = P / 2;
        constexpr int kPos = kQ * kCP / kProdThreads;
        const int pw = wave - (W::kYWaves + W::kHWaves);
        const int group = pw >> 2, pwave = pw & 3;
        const int ptid = tid - 64 * (W::kYWaves + W::kHWaves) - kProdThreads * group;
        const bool do_score = group == 0;
        const int cp = ptid % kCP, tg = ptid / kCP;
        float* const pw_l2 = scal + Lds::kBufs * kQ + pwave * 3 * kQ;   // wave i of both groups shares slot i: each writes only what it reads
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
        const auto edge_chunk = [&](int c) { return c == 0 || c * kQ + kQ - 1 > last; };
        T dtraw;
        auto issue_dt = [&](int c) { dtraw = dtp[(long long)token_of(min(c * kQ + lane, last)) * a.dt.st]; };
        // Delta and the inclusive cumulative log2-decay of position `lane` of chunk c (every producer wave runs the short
        // scan for itself); re-requests Delta for chunk cn
        auto scan_chunk = [&](int c, int cn, float& dl, float& l2) {
            dl = IoBF16::cvt(dtraw);
            issue_dt(cn);
            if (a.dt_softplus) dl = softplus(dl + dtb);
            if (c * kQ + lane > last) dl = 0.0f;
            l2 = wave_inclusive_sum(dl * a2);
        };
        // The two groups are separate code paths (not branches inside one loop) so that each keeps only its own
        // prefetch registers live.  Either way: chunk c's tiles go into buffer c & 1 from what was requested for it,
        // and every stage re-requests its inputs for chunk cn the moment it has consumed them.
        if (do_score) {
            unsigned c_src[kCopy], b_src[kCopy], c_dst[kCopy], b_dst[kCopy];
#pragma unroll
            for (int i = 0; i < kCopy; i++) {
                const int idx = i * kProdThreads + ptid;
                c_src[i] = (unsigned)(idx / (N / 8)) * a.G * N + (idx % (N / 8)) * 8;
                b_src[i] = (idx / (kQ / 8)) * kQ + (idx % (kQ / 8)) * 8;
                c_dst[i] = (idx / (N / 8)) * kRowC + (idx % (N / 8)) * 8;
                b_dst[i] = (idx / (kQ / 8)) * kRowT + (idx % (kQ / 8)) * 8;
            }
            bf16x8 ctile[kCopy], btile[kCopy];
            float4 gt[kHS];
            auto issue_score = [&](int c) {
                const float4* sc = reinterpret_cast<const float4*>(a.score_op + (((size_t)b * nchunk + c) * a.G + grp) * kScoreOp);
#pragma unroll
                for (int m = 0; m < kHS; m++) gt[m] = sc[m * kProdThreads + ptid];
            };
            auto issue_tiles = [&](int c) {
                const __bf16* csrc = a.c_rows + (((size_t)b * Lpad + (size_t)c * kQ) * a.G + grp) * N;
                const __bf16* bsrc = a.b_t + ((((size_t)b * nchunk + c) * a.G + grp) * N) * kQ;
#pragma unroll
                for (int i = 0; i < kCopy; i++) {
                    ctile[i] = *reinterpret_cast<const bf16x8*>(csrc + c_src[i]);
                    btile[i] = *reinterpret_cast<const bf16x8*>(bsrc + b_src[i]);
                }
            };
            auto finish = [&](int c, int buf, int cn) {
                float dl, l2;
                scan_chunk(c, cn, dl, l2);
                // separable decay exp(l_i - l_j) = e_i f_j around the chunk's middle unless the chunk decays too fast
                const float l2_end = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 63));
                const float l2_first = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 0));
                const float l2_mid = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), kQ / 2 - 1));
                const bool separable = l2_first - l2_end <= 100.0f;
                if (separable) {
                    pw_l2[lane] = fast_exp2(l2 - l2_mid);
                    pw_dl[lane] = fast_exp2(l2_mid - l2) * dl;
                } else {
                    pw_l2[lane] = l2;
                    pw_dl[lane] = dl;
                }
                if (pwave == 0) scal[buf * kQ + lane] = fast_exp2(l2);
                __builtin_amdgcn_wave_barrier();
                float sv[kHS][4];
#pragma unroll
                for (int m = 0; m < kHS; m++) { sv[m][0] = gt[m].x; sv[m][1] = gt[m].y; sv[m][2] = gt[m].z; sv[m][3] = gt[m].w; }
                asm volatile("" ::: "memory");
                issue_score(cn);
#pragma unroll
                for (int m = 0; m < kHS; m++) {
                    const int hs = m * kProdThreads + ptid;
                    const int bp = hs / 256, kb = (hs / 128) % 2, sl = (hs / 2) % 64, hi = hs % 2;
                    const int iblk = bp > 0, jblk = bp > 1;
                    const int i = iblk * 32 + sl % 32;
                    const int jb = jblk * 32 + 16 * kb + 8 * hi + 4 * (sl / 32);
                    const bool diagonal = iblk == jblk;
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
#pragma unroll
                for (int i = 0; i < kCopy; i++) {
                    *reinterpret_cast<bf16x8*>(&sC(buf)[c_dst[i]]) = ctile[i];
                    *reinterpret_cast<bf16x8*>(&sBT(buf)[b_dst[i]]) = btile[i];
                }
                asm volatile("" ::: "memory");
                issue_tiles(cn);
                __builtin_amdgcn_wave_barrier();   // the next chunk's scan results overwrite the tables only after these reads
            };
            issue_dt(0);
            issue_score(0);
            issue_tiles(0);
            finish(0, 0, min(1, nchunk - 1));
            lds_barrier();
            for (int c = 0; c < nchunk; c++) {
                if (c + 1 < nchunk) finish(c + 1, (c + 1) & 1, min(c + 2, nchunk - 1));
                lds_barrier();
            }
        } else {
            unsigned xraw[kPos + 3];
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
            auto finish = [&](int c, int buf, int cn) {
                float dl, l2;
                scan_chunk(c, cn, dl, l2);
                const float l2_end = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l2), 63));
                pw_wgt[lane] = fast_exp2(l2_end - l2) * dl;
                __builtin_amdgcn_wave_barrier();
                float xr[2][kPos + 3];
#pragma unroll
                for (int q = 0; q < kPos + 3; q++) {
                    xr[0][q] = __uint_as_float(xraw[q] << 16);
                    xr[1][q] = __uint_as_float(xraw[q] & 0xffff0000u);
                }
                asm volatile("" ::: "memory");
                issue_x(cn);
                if (edge_chunk(c)) {
#pragma unroll
                    for (int q = 0; q < kPos + 3; q++) {
                        const int tau = c * kQ + kPos * tg + q - 3;
                        if (tau < 0 || tau > last) xr[0][q] = xr[1][q] = 0.0f;
                    }
                    if (c == 0 && a.dir > 0 && a.tail_in && tg == 0 && a.K > 1) {
                        T cached[3][2];
#pragma unroll
                        for (int q = 0; q < 3; q++) {   // 3 - q tokens before the block; a tap beyond the conv width has a zero weight
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
                __builtin_amdgcn_wave_barrier();
            };
            issue_dt(0);
            issue_x(0);
            finish(0, 0, min(1, nchunk - 1));
            lds_barrier();
            for (int c = 0; c < nchunk; c++) {
                if (c + 1 < nchunk) finish(c + 1, (c + 1) & 1, min(c + 2, nchunk - 1));
                lds_barrier();
            }
        }
        return;
    }

    if (wave >= W::kYWaves) {
        // ------------------------------------------------------------------ h waves: row block nblk of the state
        const int nblk = wave - W::kYWaves;
        f32x16 hacc[kPB];
#pragma unroll
        for (int pb = 0; pb < kPB; pb++) {
#pragma unroll
            for (int r = 0; r < 16; r++) hacc[pb][r] = 0.0f;
            if (a.h_in) {   // registers 4q .. 4q+3: four adjacent states of channel pb*32 + cl
                const float* hrow = a.h_in + ((size_t)b * a.Dn + ch0 + pb * 32 + cl) * N + nblk * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const float4 v = *reinterpret_cast<const float4*>(hrow + 8 * q);
                    hacc[pb][4 * q] = v.x; hacc[pb][4 * q + 1] = v.y; hacc[pb][4 * q + 2] = v.z; hacc[pb][4 * q + 3] = v.w;
                }
            }
        }
        auto publish_state = [&](int which) {
#pragma unroll
            for (int pb = 0; pb < kPB; pb++) {
#pragma unroll
                for (int kb = 0; kb < 2; kb++) {
                    bf16x8 v;
#pragma unroll
                    for (int e = 0; e < 8; e++) v[e] = (__bf16)hacc[pb][8 * kb + e];
                    *reinterpret_cast<bf16x8*>(&sHT[which * Lds::kHT + (((nblk * kPB + pb) * 2 + kb) * 64 + lane) * 8]) = v;
                }
            }
        };
        publish_state(0);
        lds_barrier();
        for (int c = 0; c < nchunk; c++) {
            const int buf = c & 1;
            if (c + 1 < nchunk || a.h_out != nullptr) {   // the state after the last chunk matters only if it is committed
                const float decay_q = scal[buf * kQ + kQ - 1];
                const __bf16* b_t = sBT(buf);
                const __bf16* xw_t = sXw(buf);
#pragma unroll
                for (int pb = 0; pb < kPB; pb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) hacc[pb][r] *= decay_q;
#pragma unroll
                for (int kb = 0; kb < 4; kb++) {
                    const bf16x8 ab = *reinterpret_cast<const bf16x8*>(&b_t[(nblk * 32 + cl) * kRowT + 16 * kb + 8 * half]);
#pragma unroll
                    for (int pb = 0; pb < kPB; pb++) {
                        const bf16x8 bw = *reinterpret_cast<const bf16x8*>(&xw_t[(pb * 32 + cl) * kRowT + 16 * kb + 8 * half]);
                        hacc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab, bw, hacc[pb], 0, 0, 0);
                    }
                }
            }
            if (c + 1 < nchunk) publish_state(buf ^ 1);
            lds_barrier();
        }
        if (a.h_out) {
#pragma unroll
            for (int pb = 0; pb < kPB; pb++) {
                float* hrow = a.h_out + ((size_t)b * a.Dn + ch0 + pb * 32 + cl) * N + nblk * 32 + 4 * half;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    *reinterpret_cast<float4*>(hrow + 8 * q) =
                        make_float4(hacc[pb][4 * q], hacc[pb][4 * q + 1], hacc[pb][4 * q + 2], hacc[pb][4 * q + 3]);
            }
        }
        return;
    }

    // ---------------------------------------------------------------------- y waves: one 32 x 32 block of the output
    auto walk = [&](auto mode_c) {
        constexpr int kMode = decltype(mode_c)::value;
        constexpr bool need_z = kMode != kSsdPartialRaw;
        constexpr bool need_p = kMode == kSsdFinalAdd || kMode == kSsdFinalAddRaw;
        constexpr bool parks = kMode == kSsdPartialRaw || kMode == kSsdPartial;
        const int iblk = wave / kPB, pblk = wave % kPB;
        const int po = pblk * 32 + cl;
        const int icol = iblk * 32 + cl;
        const int i0 = iblk * 32 + 4 * half;
        auto row_k = [](int r) { return 8 * (r / 4) + (r % 4); };
        const float dval = a.D[a.d_per_head ? head : ch0 + po];
        // rows of a chunk that lies inside the sequence, relative to the chunk's lowest-address token: the row of
        // accumulator register 4q + e is group[q] (in the lane offset) plus step[e] (a scalar offset), see the header
        const int fwd = a.dir > 0;
        const unsigned zs = (unsigned)a.z.st * 2u, os = (unsigned)a.out_st * 2u, ps = (unsigned)a.Dn * 2u;
        unsigned zoff[4], ooff[4], poff[4];
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const unsigned rows = (unsigned)(fwd ? iblk * 32 + 8 * q + 4 * half : 56 - iblk * 32 - 8 * q + 4 * (1 - half));
            zoff[q] = rows * zs + 2u * (unsigned)po;
            ooff[q] = rows * os + 2u * (unsigned)po;
            poff[q] = rows * ps + 2u * (unsigned)po;
        }
        // (scalar registers by construction: left to the compiler the direction select lands in vector registers and
        // every access loops over the lanes to read its offset back)
        int zstep[4], ostep[4], pstep[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int m = fwd ? e : 3 - e;
            zstep[e] = __builtin_amdgcn_readfirstlane(m * (int)zs);
            ostep[e] = __builtin_amdgcn_readfirstlane(m * (int)os);
            pstep[e] = __builtin_amdgcn_readfirstlane(m * (int)ps);
        }
        const T* const zhead = (const T*)a.z.p + (size_t)b * a.z.sb + ch0;
        const T* const phead = (const T*)a.partial + (size_t)b * a.L * a.Dn + ch0;   // the parked result is bf16
        T* const ohead = (T*)a.out + (size_t)b * a.out_sb + a.out_ch_off + ch0;
        auto chunk_low_token = [&](int c) { return (long long)(fwd ? c * kQ : last - (c * kQ + kQ - 1)); };

        T zraw[16], praw[16];
        auto issue_gate = [&](int c) {
            if (c * kQ + kQ - 1 <= last) {
                const long long t0 = chunk_low_token(c);
                const Rsrc zr = raw_range(zhead + t0 * a.z.st), pr = raw_range(phead + t0 * a.Dn);
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    if constexpr (need_z) zraw[r] = IoBF16::ld_raw(zr, zoff[r / 4], zstep[r % 4]);
                    if constexpr (need_p) praw[r] = IoBF16::ld_raw(pr, poff[r / 4], pstep[r % 4]);
                }
            } else {
                const int tau0 = c * kQ + i0;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const long long t = token_of(min(tau0 + row_k(r), last));
                    if constexpr (need_z) zraw[r] = zhead[t * a.z.st + po];
                    if constexpr (need_p) praw[r] = phead[t * a.Dn + po];
                }
            }
        };
        bool state_nonzero = a.h_in != nullptr;
        issue_gate(0);
        lds_barrier();
        for (int c = 0; c < nchunk; c++) {
            const int buf = c & 1;
            const float* el = scal + buf * kQ;
            const __bf16* xc_t = sXc(buf);
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
            if (state_nonzero) {
                const __bf16* c_t = sC(buf);
                const __bf16* h_t = sHT + buf * Lds::kHT;
#pragma unroll
                for (int nb = 0; nb < kNB; nb++) {
#pragma unroll
                    for (int kb = 0; kb < 2; kb++) {
                        bf16x8 ac;
#pragma unroll
                        for (int jj = 0; jj < 2; jj++) {
                            const bf16x4 v = *reinterpret_cast<const bf16x4*>(&c_t[icol * kRowC + nb * 32 + 16 * kb + 8 * jj + 4 * half]);
#pragma unroll
                            for (int e = 0; e < 4; e++) ac[4 * jj + e] = v[e];
                        }
                        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(&h_t[(((nb * kPB + pblk) * 2 + kb) * 64 + lane) * 8]);
                        y2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ac, bh, y2, 0, 0, 0);
                    }
                }
            }
            // epilogue: inter-chunk term, skip term, gate, combine; all 16 results first, then the stores
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
                        const float pv = need_p ? IoBF16::cvt(praw[r]) : 0.0f;
                        res[r] = kMode == kSsdFinalAddRaw ? (y + pv) * zg : need_p ? y * zg + pv : y * zg;
                    }
                }
            }
            if (c * kQ + kQ - 1 <= last) {
                const long long t0 = chunk_low_token(c);
                const Rsrc orr = raw_range(parks ? (T*)phead + t0 * a.Dn : ohead + t0 * a.out_st);
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    if constexpr (parks) IoBF16::st_raw(orr, poff[r / 4], pstep[r % 4], res[r]);
                    else IoBF16::st_raw(orr, ooff[r / 4], ostep[r % 4], res[r]);
                }
            } else {
                const int tau0 = c * kQ + i0;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int tau = tau0 + row_k(r);
                    if (tau <= last) {
                        const long long t = token_of(tau);
                        if constexpr (parks) IoBF16::st((T*)phead + t * a.Dn + po, res[r]);
                        else IoBF16::st(ohead + t * a.out_st + po, res[r]);
                    }
                }
            }
            if (c + 1 < nchunk) issue_gate(c + 1);
            state_nonzero = true;
            lds_barrier();
        }
    };
    switch (a.mode) {
        case kSsdFinalOnly: walk(std::integral_constant<int, kSsdFinalOnly>{}); break;
        case kSsdPartial: walk(std::integral_constant<int, kSsdPartial>{}); break;
        case kSsdPartialRaw: walk(std::integral_constant<int, kSsdPartialRaw>{}); break;
        case kSsdFinalAdd: walk(std::integral_constant<int, kSsdFinalAdd>{}); break;
        default: walk(std::integral_constant<int, kSsdFinalAddRaw>{}); break;
    }
}

}  // namespace bm
