/*
 * bimamba_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, sequential fp64 CPU statement of what the bidirectional Mamba
 * mixer inner path computes: depthwise short conv + SiLU, the selective
 * state-space recurrence run left-to-right and right-to-left, the SiLU(z) gate
 * and the combine of the two directions (paper Sec. 3.2 eqs. 4-6: forward
 * recurrence i = 1..L, reverse recurrence i = L..1, additive fusion), plus the
 * state-carrying block variant (paper Sec. 4.3: forward state propagated across
 * blocks, right-to-left updates confined to the current block).
 *
 * It shares no code, header, table or helper with the HIP library.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Precision: inputs arrive as float arrays (values exactly representable in the
 * I/O dtype, bf16 or fp32); every operation below is done in double; nothing is
 * rounded on the way out.  No blocking, chunking, fusion or reordering: one
 * (batch, channel) row at a time, one token at a time, one state at a time.
 *
 * Pins of the gradients (tests/test_oracle_bwd_pins.py): central finite differences of orc_bimamba_fwd with
 * Richardson extrapolation, for every input and parameter element on small shapes; automatic differentiation of the
 * same definition written with a tensor library's differentiable ops.
 *
 * Pins (tests/test_oracle_pins.py): L=1 closed form, A=0 weighted cumulative
 * sum, geometric closed form, brute-force y = M x for L<=16, reverse ==
 * flip(forward(flip)), library depthwise convolution, split-anywhere state
 * carry, block variant == slice of the full scan, ADD == sum of SEPARATE halves.
 *
 * Layout of every activation tensor: token-major, channel fastest, contiguous:
 *   x, z  [batch, L, d_inner]          dt [batch, L, n_heads]
 *   B, C  [batch, L, n_groups, d_state]
 *   out   [batch, L, n_sel] (ADD)   or [batch, L, 2, n_sel] (SEPARATE)
 * where n_sel = number of selected channels (all of d_inner when sel == NULL).
 * Channel d belongs to head d / (d_inner/n_heads); head h to group
 * h / (n_heads/n_groups).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int batch, seqlen, d_inner, d_state, n_heads, n_groups, d_conv;
    int a_kind;      /* 0: A[n_heads][d_state]   1: A[n_heads] (one scalar per head) */
    int d_kind;      /* 0: D[d_inner]            1: D[n_heads] */
    int dt_softplus; /* 0: dt is Delta itself    1: Delta = softplus(dt + dt_bias[head]) */
    int conv_bc;     /* 0: conv over x only      1: conv over x | B | C channels */
    int combine;     /* 0: out = g_f + g_b       1: out = [g_f | g_b] */
} orc_desc;

/* conv_w [conv_ch][d_conv], conv_b [conv_ch] or NULL, conv_ch = d_inner (+ 2*n_groups*d_state) */
typedef struct { const float *conv_w, *conv_b, *A, *D, *dt_bias; } orc_params;
typedef struct { const float *x, *z, *dt, *B, *C; } orc_inputs;

static double silu(double v) { return v / (1.0 + exp(-v)); }
static double softplus(double v) { return v > 0.0 ? v + log1p(exp(-v)) : log1p(exp(v)); }

/*
 * Depthwise conv of width K followed by SiLU, for one channel, in one direction.
 * dir=+1 (causal):      pre[t] = b + sum_k w[k] * src[t - (K-1-k)]
 * dir=-1 (anti-causal): pre[t] = b + sum_k w[k] * src[t + (K-1-k)]
 * so w[K-1] always multiplies the current token.  Tokens outside [0,L) are zero,
 * except that on the causal side `left` (K-1 values, oldest first: left[j] is
 * the token at index j-(K-1)) supplies the tokens before the block when given.
 */
static void conv_silu_1ch(const float *src, long stride, int L, int K, const float *w, double bias,
                          int dir, const double *left, double *dst)
{
    for (int t = 0; t < L; t++) {
        double acc = bias;
        for (int k = 0; k < K; k++) {
            int back = K - 1 - k;              /* how many tokens "behind" in scan order */
            int idx = t - dir * back;
            double v;
            if (idx >= 0 && idx < L) v = (double)src[(long)idx * stride];
            else if (idx < 0 && dir > 0 && left) v = left[idx + (K - 1)];
            else v = 0.0;
            acc += (double)w[k] * v;
        }
        dst[t] = silu(acc);
    }
}

/*
 * The recurrence for one (batch, channel) row in one direction (eq. 4 for
 * dir=+1, eq. 5 for dir=-1), in the concrete selective-scan form
 *   h_t[n] = exp(Delta_t * A[n]) * h_prev[n] + Delta_t * B_t[n] * xc_t
 *   y_t    = sum_n C_t[n] * h_t[n] + D * xc_t
 * h starts from h0 (NULL = zero) and its final value is written to h_end when
 * that is not NULL.  Bc, Cc: [L][bc_stride] doubles, N used entries per token.
 */
static void scan_row(int L, int N, int dir, const double *xc, const double *delta,
                     const double *Bc, const double *Cc, long bc_stride,
                     const double *Arow /* N entries */, double Dval,
                     const double *h0, double *h_end, double *y)
{
    double *h = (double *)malloc(sizeof(double) * (size_t)N);
    for (int n = 0; n < N; n++) h[n] = h0 ? h0[n] : 0.0;
    int t = dir > 0 ? 0 : L - 1;
    for (int step = 0; step < L; step++, t += dir) {
        double acc = 0.0;
        const double *Bt = Bc + (long)t * bc_stride, *Ct = Cc + (long)t * bc_stride;
        for (int n = 0; n < N; n++) {
            h[n] = exp(delta[t] * Arow[n]) * h[n] + delta[t] * Bt[n] * xc[t];
            acc += Ct[n] * h[n];
        }
        y[t] = acc + Dval * xc[t];
    }
    if (h_end) for (int n = 0; n < N; n++) h_end[n] = h[n];
    free(h);
}

/*
 * One direction of the mixer for one batch element, on the selected channels:
 * conv+SiLU (x and, if conv_bc, B and C), Delta, scan, gate.  g: [L][n_sel].
 * h0 / h_end: [d_inner][N] indexed by true channel (may be NULL).
 * tail: [(K-1)][tail_ch] doubles for this batch element or NULL (causal side only).
 */
static void one_direction(const orc_desc *d, const orc_params *p, const orc_inputs *in, int b, int dir,
                          const int *sel, int n_sel, const double *h0, double *h_end,
                          const double *tail, double *g, long g_stride)
{
    const int L = d->seqlen, Dn = d->d_inner, N = d->d_state, H = d->n_heads, G = d->n_groups, K = d->d_conv;
    const int P = Dn / H, HG = H / G, GN = G * N;
    const int tail_ch = Dn + (d->conv_bc ? 2 * GN : 0);
    const float *xb = in->x + (long)b * L * Dn, *zb = in->z + (long)b * L * Dn;
    const float *dtb = in->dt + (long)b * L * H;
    const float *Bb = in->B + (long)b * L * GN, *Cb = in->C + (long)b * L * GN;

    /* B and C as the scan sees them: raw, or conv+SiLU'd like x (channel order x | B | C) */
    double *Bc = (double *)malloc(sizeof(double) * (size_t)L * GN);
    double *Cc = (double *)malloc(sizeof(double) * (size_t)L * GN);
    if (d->conv_bc) {
        double *col = (double *)malloc(sizeof(double) * (size_t)L);
        double left[8];
        for (int j = 0; j < GN; j++) {
            for (int which = 0; which < 2; which++) {
                int ch = Dn + which * GN + j;
                const float *src = (which ? Cb : Bb) + j;
                if (tail) for (int q = 0; q < K - 1; q++) left[q] = tail[(long)q * tail_ch + ch];
                conv_silu_1ch(src, GN, L, K, p->conv_w + (long)ch * K, p->conv_b ? (double)p->conv_b[ch] : 0.0,
                              dir, tail ? left : NULL, col);
                double *dstm = which ? Cc : Bc;
                for (int t = 0; t < L; t++) dstm[(long)t * GN + j] = col[t];
            }
        }
        free(col);
    } else {
        for (long i = 0; i < (long)L * GN; i++) { Bc[i] = (double)Bb[i]; Cc[i] = (double)Cb[i]; }
    }

#pragma omp parallel
    {
        double *xc = (double *)malloc(sizeof(double) * (size_t)L);
        double *delta = (double *)malloc(sizeof(double) * (size_t)L);
        double *y = (double *)malloc(sizeof(double) * (size_t)L);
        double *Arow = (double *)malloc(sizeof(double) * (size_t)N);
        double left[8];
#pragma omp for schedule(dynamic, 4)
        for (int s = 0; s < n_sel; s++) {
            const int ch = sel ? sel[s] : s;
            const int head = ch / P, grp = head / HG;
            if (tail) for (int q = 0; q < K - 1; q++) left[q] = tail[(long)q * tail_ch + ch];
            conv_silu_1ch(xb + ch, Dn, L, K, p->conv_w + (long)ch * K, p->conv_b ? (double)p->conv_b[ch] : 0.0,
                          dir, tail ? left : NULL, xc);
            for (int t = 0; t < L; t++) {
                double v = (double)dtb[(long)t * H + head];
                delta[t] = d->dt_softplus ? softplus(v + (p->dt_bias ? (double)p->dt_bias[head] : 0.0)) : v;
            }
            for (int n = 0; n < N; n++)
                Arow[n] = d->a_kind == 0 ? (double)p->A[(long)head * N + n] : (double)p->A[head];
            const double Dval = d->d_kind == 0 ? (double)p->D[ch] : (double)p->D[head];
            scan_row(L, N, dir, xc, delta, Bc + (long)grp * N, Cc + (long)grp * N, GN, Arow, Dval,
                     h0 ? h0 + (long)ch * N : NULL, h_end ? h_end + (long)ch * N : NULL, y);
            for (int t = 0; t < L; t++)
                g[(long)t * g_stride + s] = y[t] * silu((double)zb[(long)t * Dn + ch]);
        }
        free(xc); free(delta); free(y); free(Arow);
    }
    free(Bc); free(Cc);
}

static void combine_into(const orc_desc *d, int n_sel, const double *gf, const double *gb, double *outb)
{
    const int L = d->seqlen;
    for (int t = 0; t < L; t++)
        for (int s = 0; s < n_sel; s++) {
            if (d->combine == 0) outb[(long)t * n_sel + s] = gf[(long)t * n_sel + s] + gb[(long)t * n_sel + s];
            else {
                outb[((long)t * 2 + 0) * n_sel + s] = gf[(long)t * n_sel + s];
                outb[((long)t * 2 + 1) * n_sel + s] = gb[(long)t * n_sel + s];
            }
        }
}

/*
 * Full-sequence bidirectional mixer path (eqs. 4-6).  in_b may equal in_f
 * (both directions read the same activations) and pb may equal pf (tied weights).
 * sel: n_sel channel indices to evaluate, or NULL for all d_inner channels.
 * Returns 0, or -1 on a shape the definition does not cover.
 */
int orc_bimamba_fwd(const orc_desc *d, const orc_params *pf, const orc_params *pb,
                    const orc_inputs *in_f, const orc_inputs *in_b,
                    const int *sel, int n_sel, double *out)
{
    if (d->batch < 0 || d->seqlen < 0 || d->d_inner < 1 || d->d_state < 1 || d->n_heads < 1 || d->n_groups < 1) return -1;
    if (d->d_inner % d->n_heads || d->n_heads % d->n_groups || d->d_conv < 1 || d->d_conv > 8) return -1;
    if (!sel) n_sel = d->d_inner;
    const int L = d->seqlen;
    const long per_b = (long)L * n_sel * (d->combine ? 2 : 1);
    double *gf = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * n_sel);
    double *gb = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * n_sel);
    for (int b = 0; b < d->batch; b++) {
        one_direction(d, pf, in_f, b, +1, sel, n_sel, NULL, NULL, NULL, gf, n_sel);
        one_direction(d, pb, in_b, b, -1, sel, n_sel, NULL, NULL, NULL, gb, n_sel);
        combine_into(d, n_sel, gf, gb, out + (long)b * per_b);
    }
    free(gf); free(gb);
    return 0;
}

/*
 * Block variant (Sec. 4.3).  d->seqlen is the block length.  The forward
 * direction resumes from h_in [batch][d_inner][d_state] (NULL = zero) and, for
 * its causal conv, from tail_in [batch][d_conv-1][tail_ch] (NULL = zero), the
 * raw pre-conv tokens that precede the block, oldest first; tail_ch = d_inner
 * (+ 2*n_groups*d_state when conv_bc, channel order x | B | C).  The reverse
 * direction starts from zero at the block's right edge and sees zeros beyond it.
 * h_out (may be NULL): forward state after the block's last token.
 * tail_out (may be NULL): the last d_conv-1 raw tokens of tail_in || block.
 */
int orc_bimamba_block_fwd(const orc_desc *d, const orc_params *pf, const orc_params *pb,
                          const orc_inputs *in_f, const orc_inputs *in_b,
                          const double *h_in, const double *tail_in,
                          const int *sel, int n_sel, double *out, double *h_out, double *tail_out)
{
    if (d->batch < 0 || d->seqlen < 0 || d->d_inner < 1 || d->d_state < 1 || d->n_heads < 1 || d->n_groups < 1) return -1;
    if (d->d_inner % d->n_heads || d->n_heads % d->n_groups || d->d_conv < 1 || d->d_conv > 8) return -1;
    if (!sel) n_sel = d->d_inner;
    const int L = d->seqlen, Dn = d->d_inner, N = d->d_state, K = d->d_conv, GN = d->n_groups * N;
    const int tail_ch = Dn + (d->conv_bc ? 2 * GN : 0);
    const long per_b = (long)L * n_sel * (d->combine ? 2 : 1);
    double *gf = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * n_sel);
    double *gb = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * n_sel);
    for (int b = 0; b < d->batch; b++) {
        const double *h0 = h_in ? h_in + (long)b * Dn * N : NULL;
        double *he = h_out ? h_out + (long)b * Dn * N : NULL;
        const double *tl = tail_in ? tail_in + (long)b * (K - 1) * tail_ch : NULL;
        if (he && L == 0) for (long i = 0; i < (long)Dn * N; i++) he[i] = h0 ? h0[i] : 0.0;
        one_direction(d, pf, in_f, b, +1, sel, n_sel, h0, he, tl, gf, n_sel);
        one_direction(d, pb, in_b, b, -1, sel, n_sel, NULL, NULL, NULL, gb, n_sel);
        combine_into(d, n_sel, gf, gb, out + (long)b * per_b);
        if (tail_out) {
            /* stream = tail_in (K-1 tokens) followed by the block's L raw tokens; keep the last K-1 */
            double *to = tail_out + (long)b * (K - 1) * tail_ch;
            for (int q = 0; q < K - 1; q++) {
                int pos = L + q;                       /* index in the stream of length (K-1)+L */
                for (int c = 0; c < tail_ch; c++) {
                    double v;
                    if (pos < K - 1) v = tl ? tl[(long)pos * tail_ch + c] : 0.0;
                    else {
                        int t = pos - (K - 1);
                        if (c < Dn) v = (double)in_f->x[((long)b * L + t) * Dn + c];
                        else if (c < Dn + GN) v = (double)in_f->B[((long)b * L + t) * GN + (c - Dn)];
                        else v = (double)in_f->C[((long)b * L + t) * GN + (c - Dn - GN)];
                    }
                    to[(long)q * tail_ch + c] = v;
                }
            }
        }
    }
    free(gf); free(gb);
    return 0;
}

/* Single-direction entry used by the pins (forward-only scans, explicit h0 / h_end). */
int orc_one_direction(const orc_desc *d, const orc_params *p, const orc_inputs *in, int dir,
                      const double *h_in, const double *tail_in, double *g, double *h_out)
{
    const int L = d->seqlen, Dn = d->d_inner, N = d->d_state, K = d->d_conv;
    const int tail_ch = Dn + (d->conv_bc ? 2 * d->n_groups * N : 0);
    if (d->d_inner % d->n_heads || d->n_heads % d->n_groups || d->d_conv < 1 || d->d_conv > 8) return -1;
    for (int b = 0; b < d->batch; b++) {
        double *he = h_out ? h_out + (long)b * Dn * N : NULL;
        const double *h0 = h_in ? h_in + (long)b * Dn * N : NULL;
        if (he && L == 0) for (long i = 0; i < (long)Dn * N; i++) he[i] = h0 ? h0[i] : 0.0;
        one_direction(d, p, in, b, dir, NULL, Dn, h0, he,
                      tail_in ? tail_in + (long)b * (K - 1) * tail_ch : NULL,
                      g + (long)b * L * Dn, Dn);
    }
    return 0;
}

/*
 * ---- Gradients (the paper trains these models, App. A.2; it gives no backward algorithm, so this is the chain rule
 * of the forward definition above, one row, one token, one state at a time, in the reverse of the scan order).
 *
 * For one direction and one (batch, channel) row, with t running over the scan order and t- the step before t:
 *   pre_t = cb + sum_k w_k x_{t - dir*(K-1-k)}      xc_t = silu(pre_t)
 *   delta_t = dt_t  or  softplus(dt_t + bias)       a_t[n] = exp(delta_t A[n])
 *   h_t[n] = a_t[n] h_{t-}[n] + delta_t B_t[n] xc_t
 *   y_t = sum_n C_t[n] h_t[n] + D xc_t              g_t = y_t silu(z_t)
 * Given dg_t (the upstream gradient of g_t):
 *   dz_t += dg_t y_t silu'(z_t)                     dy_t = dg_t silu(z_t)
 *   dh_t[n] = C_t[n] dy_t + a_{t+}[n] dh_{t+}[n]    (t+ the step after t; zero after the last step)
 *   dC_t[n] += dy_t h_t[n]                          dD += dy_t xc_t
 *   dA[n] += dh_t[n] h_{t-}[n] a_t[n] delta_t       dB_t[n] += dh_t[n] delta_t xc_t
 *   ddelta_t = sum_n dh_t[n] (h_{t-}[n] a_t[n] A[n] + B_t[n] xc_t)
 *   dxc_t = D dy_t + sum_n dh_t[n] delta_t B_t[n]   dpre_t = dxc_t silu'(pre_t)
 *   ddt_t += ddelta_t (times sigmoid(dt_t + bias) with softplus, which also feeds dbias)
 *   dcb += dpre_t;  dw_k += dpre_t x_{t - dir*(K-1-k)};  dx_{t - dir*(K-1-k)} += w_k dpre_t
 * With conv_bc, B_t and C_t are themselves silu(conv(raw)) and their gradients go through the same conv rule.
 * All outputs are accumulated into (+=): the caller zeroes them and may pass the same arrays for both directions.
 */
typedef struct { double *dx, *dz, *ddt, *dB, *dC; } orc_input_grads;   /* dx, dz [batch][L][n_sel]; ddt [batch][L][H]; dB, dC [batch][L][G*N] */
typedef struct { double *dconv_w, *dconv_b, *dA, *dD, *ddt_bias; } orc_param_grads; /* shaped like the parameters */

static double dsilu(double v) { const double s = 1.0 / (1.0 + exp(-v)); return s * (1.0 + v * (1.0 - s)); }
static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

/* gradient of silu(conv(src)) for one channel: dval[t] is the gradient of the conv+SiLU output at t */
static void conv_silu_1ch_bwd(const float *src, long stride, int L, int K, const float *w, double bias, int dir,
                              const double *dval, double *dsrc, long dstride, double *dw, double *db)
{
    for (int t = 0; t < L; t++) {
        double acc = bias;
        for (int k = 0; k < K; k++) {
            int idx = t - dir * (K - 1 - k);
            if (idx >= 0 && idx < L) acc += (double)w[k] * (double)src[(long)idx * stride];
        }
        const double dpre = dval[t] * dsilu(acc);
        if (db) *db += dpre;
        for (int k = 0; k < K; k++) {
            int idx = t - dir * (K - 1 - k);
            if (idx >= 0 && idx < L) {
                dw[k] += dpre * (double)src[(long)idx * stride];
                dsrc[(long)idx * dstride] += (double)w[k] * dpre;
            }
        }
    }
}

static void one_direction_bwd(const orc_desc *d, const orc_params *p, const orc_inputs *in, int b, int dir,
                              const int *sel, int n_sel, const double *dg, long dg_stride,
                              const orc_input_grads *gi, const orc_param_grads *gp)
{
    const int L = d->seqlen, Dn = d->d_inner, N = d->d_state, H = d->n_heads, G = d->n_groups, K = d->d_conv;
    const int P = Dn / H, HG = H / G, GN = G * N;
    const float *xb = in->x + (long)b * L * Dn, *zb = in->z + (long)b * L * Dn;
    const float *dtb = in->dt + (long)b * L * H;
    const float *Bb = in->B + (long)b * L * GN, *Cb = in->C + (long)b * L * GN;
    double *Bc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * GN);
    double *Cc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * GN);
    double *dBc = (double *)calloc((size_t)(L > 0 ? L : 1) * GN, sizeof(double));
    double *dCc = (double *)calloc((size_t)(L > 0 ? L : 1) * GN, sizeof(double));
    double *col = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    if (d->conv_bc) {
        for (int j = 0; j < GN; j++)
            for (int which = 0; which < 2; which++) {
                int ch = Dn + which * GN + j;
                conv_silu_1ch((which ? Cb : Bb) + j, GN, L, K, p->conv_w + (long)ch * K,
                              p->conv_b ? (double)p->conv_b[ch] : 0.0, dir, NULL, col);
                for (int t = 0; t < L; t++) (which ? Cc : Bc)[(long)t * GN + j] = col[t];
            }
    } else {
        for (long i = 0; i < (long)L * GN; i++) { Bc[i] = (double)Bb[i]; Cc[i] = (double)Cb[i]; }
    }
    double *xc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *delta = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *dxc = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *hall = (double *)malloc(sizeof(double) * (size_t)(L + 1) * N);   /* hall[step+1] = state after scan step `step` */
    double *dh = (double *)malloc(sizeof(double) * (size_t)N);
    double *Arow = (double *)malloc(sizeof(double) * (size_t)N);
    for (int s = 0; s < n_sel; s++) {
        const int ch = sel ? sel[s] : s;
        const int head = ch / P, grp = head / HG;
        const double bias = (d->dt_softplus && p->dt_bias) ? (double)p->dt_bias[head] : 0.0;
        conv_silu_1ch(xb + ch, Dn, L, K, p->conv_w + (long)ch * K, p->conv_b ? (double)p->conv_b[ch] : 0.0, dir, NULL, xc);
        for (int t = 0; t < L; t++) {
            double v = (double)dtb[(long)t * H + head];
            delta[t] = d->dt_softplus ? softplus(v + bias) : v;
        }
        for (int n = 0; n < N; n++) Arow[n] = d->a_kind == 0 ? (double)p->A[(long)head * N + n] : (double)p->A[head];
        const double Dval = d->d_kind == 0 ? (double)p->D[ch] : (double)p->D[head];
        /* forward, keeping every state */
        for (int n = 0; n < N; n++) hall[n] = 0.0;
        {
            int t = dir > 0 ? 0 : L - 1;
            for (int step = 0; step < L; step++, t += dir) {
                const double *Bt = Bc + (long)t * GN + (long)grp * N;
                for (int n = 0; n < N; n++)
                    hall[(long)(step + 1) * N + n] = exp(delta[t] * Arow[n]) * hall[(long)step * N + n] + delta[t] * Bt[n] * xc[t];
            }
        }
        /* backward, last scan step first */
        for (int n = 0; n < N; n++) dh[n] = 0.0;
        {
            int t = dir > 0 ? L - 1 : 0;
            for (int step = L - 1; step >= 0; step--, t -= dir) {
                const double *Bt = Bc + (long)t * GN + (long)grp * N, *Ct = Cc + (long)t * GN + (long)grp * N;
                double *dBt = dBc + (long)t * GN + (long)grp * N, *dCt = dCc + (long)t * GN + (long)grp * N;
                const double *hcur = hall + (long)(step + 1) * N, *hprev = hall + (long)step * N;
                const double zv = (double)zb[(long)t * Dn + ch];
                const double dgt = dg[(long)t * dg_stride + s];
                double y = Dval * xc[t];
                for (int n = 0; n < N; n++) y += Ct[n] * hcur[n];
                gi->dz[((long)b * L + t) * n_sel + s] += dgt * y * dsilu(zv);
                const double dy = dgt * silu(zv);
                double ddelta = 0.0, dxct = Dval * dy;
                if (gp->dD) gp->dD[d->d_kind == 0 ? ch : head] += dy * xc[t];
                for (int n = 0; n < N; n++) {
                    const double a = exp(delta[t] * Arow[n]);
                    dh[n] += Ct[n] * dy;
                    dCt[n] += dy * hcur[n];
                    if (gp->dA) gp->dA[d->a_kind == 0 ? (long)head * N + n : head] += dh[n] * hprev[n] * a * delta[t];
                    dBt[n] += dh[n] * delta[t] * xc[t];
                    ddelta += dh[n] * (hprev[n] * a * Arow[n] + Bt[n] * xc[t]);
                    dxct += dh[n] * delta[t] * Bt[n];
                    dh[n] *= a;
                }
                if (d->dt_softplus) {
                    const double sg = sigmoid((double)dtb[(long)t * H + head] + bias);
                    gi->ddt[((long)b * L + t) * H + head] += ddelta * sg;
                    if (gp->ddt_bias) gp->ddt_bias[head] += ddelta * sg;
                } else {
                    gi->ddt[((long)b * L + t) * H + head] += ddelta;
                }
                dxc[t] = dxct;
            }
        }
        conv_silu_1ch_bwd(xb + ch, Dn, L, K, p->conv_w + (long)ch * K, p->conv_b ? (double)p->conv_b[ch] : 0.0, dir,
                          dxc, gi->dx + (long)b * L * n_sel + s, n_sel, gp->dconv_w + (long)ch * K,
                          gp->dconv_b ? gp->dconv_b + ch : NULL);
    }
    /* B and C: straight through, or back through their own conv + SiLU */
    if (d->conv_bc) {
        for (int j = 0; j < GN; j++)
            for (int which = 0; which < 2; which++) {
                int ch = Dn + which * GN + j;
                for (int t = 0; t < L; t++) col[t] = (which ? dCc : dBc)[(long)t * GN + j];
                conv_silu_1ch_bwd((which ? Cb : Bb) + j, GN, L, K, p->conv_w + (long)ch * K,
                                  p->conv_b ? (double)p->conv_b[ch] : 0.0, dir, col,
                                  (which ? gi->dC : gi->dB) + (long)b * L * GN + j, GN, gp->dconv_w + (long)ch * K,
                                  gp->dconv_b ? gp->dconv_b + ch : NULL);
            }
    } else {
        for (long i = 0; i < (long)L * GN; i++) {
            gi->dB[(long)b * L * GN + i] += dBc[i];
            gi->dC[(long)b * L * GN + i] += dCc[i];
        }
    }
    free(Bc); free(Cc); free(dBc); free(dCc); free(col); free(xc); free(delta); free(dxc); free(hall); free(dh); free(Arow);
}

/*
 * Gradients of the full-sequence path (orc_bimamba_fwd) given dout, the gradient of its output:
 * dout [batch][L][n_sel] (ADD: both directions receive it) or [batch][L][2][n_sel] (SEPARATE: half 0 forward).
 * gin_f / gin_b and gpf / gpb may point at the same arrays when the directions share inputs or parameters.
 */
int orc_bimamba_bwd(const orc_desc *d, const orc_params *pf, const orc_params *pb,
                    const orc_inputs *in_f, const orc_inputs *in_b, const int *sel, int n_sel, const double *dout,
                    const orc_input_grads *gin_f, const orc_input_grads *gin_b,
                    const orc_param_grads *gpf, const orc_param_grads *gpb)
{
    if (d->batch < 0 || d->seqlen < 0 || d->d_inner < 1 || d->d_state < 1 || d->n_heads < 1 || d->n_groups < 1) return -1;
    if (d->d_inner % d->n_heads || d->n_heads % d->n_groups || d->d_conv < 1 || d->d_conv > 8) return -1;
    if (!sel) n_sel = d->d_inner;
    const int L = d->seqlen;
    const long per_b = (long)L * n_sel * (d->combine ? 2 : 1);
    const long stride = (long)n_sel * (d->combine ? 2 : 1);
    for (int b = 0; b < d->batch; b++) {
        const double *dob = dout + (long)b * per_b;
        one_direction_bwd(d, pf, in_f, b, +1, sel, n_sel, dob, stride, gin_f, gpf);
        one_direction_bwd(d, pb, in_b, b, -1, sel, n_sel, dob + (d->combine ? n_sel : 0), stride, gin_b, gpb);
    }
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}
