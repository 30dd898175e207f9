/*
 * san_check.c -- TEST INFRASTRUCTURE: walks the oracle's entry points over edge shapes in a build with
 * AddressSanitizer and UBSan (oracle/build.py links it against bimamba_oracle.c).  Every buffer is allocated at its
 * exact size (outputs: one spare element), so an index past the end of any input tensor or before the start of any
 * tensor is a sanitizer report and a non-zero exit.  Prints one
 * checksum per case; tests/test_oracle_sanitized.py compares them with the plain build's results on the same inputs.
 *
 * Inputs come from a fixed linear congruential sequence (no arithmetic of the method here): the test regenerates the
 * same values in Python.
 */
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int batch, seqlen, d_inner, d_state, n_heads, n_groups, d_conv;
    int a_kind, d_kind, dt_softplus, conv_bc, combine;
} orc_desc;
typedef struct { const float *conv_w, *conv_b, *A, *D, *dt_bias; } orc_params;
typedef struct { const float *x, *z, *dt, *B, *C; } orc_inputs;

int orc_bimamba_fwd(const orc_desc *d, const orc_params *pf, const orc_params *pb, const orc_inputs *in_f,
                    const orc_inputs *in_b, const int *sel, int n_sel, double *out);
int orc_bimamba_block_fwd(const orc_desc *d, const orc_params *pf, const orc_params *pb, const orc_inputs *in_f,
                          const orc_inputs *in_b, const double *h_in, const double *tail_in, const int *sel, int n_sel,
                          double *out, double *h_out, double *tail_out);
int orc_one_direction(const orc_desc *d, const orc_params *p, const orc_inputs *in, int dir, const double *h_in,
                      const double *tail_in, double *g, double *h_out);

static unsigned long long lcg_state;
static float next_value(void)   /* multiples of 1/64 in [-2, 2): exact in every I/O dtype */
{
    lcg_state = lcg_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((int)((lcg_state >> 33) % 256) - 128) / 64.0f;
}
static float *fill(size_t n, int positive, int negative)
{
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    for (size_t i = 0; i < n; i++) {
        float v = next_value();
        if (positive) v = (v < 0 ? -v : v) * 0.05f + 0.001f;
        if (negative) v = -((v < 0 ? -v : v) + 0.25f);
        p[i] = v;
    }
    return p;
}
static double checksum(const double *p, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; i++) s += p[i] * (double)(1 + (i % 7));
    return s;
}

static int run_case(int id, orc_desc d, int use_sel, int with_state)
{
    const int GN = d.n_groups * d.d_state, cc = d.d_inner + (d.conv_bc ? 2 * GN : 0);
    const size_t tokens = (size_t)d.batch * d.seqlen;
    lcg_state = 1000 + id;
    orc_params p[2];
    float *owned[64]; int n_owned = 0;
#define KEEP(ptr) (owned[n_owned++] = (ptr))
    for (int s = 0; s < 2; s++) {
        p[s].conv_w = KEEP(fill((size_t)cc * d.d_conv, 0, 0));
        p[s].conv_b = (id % 3 == 0) ? NULL : KEEP(fill(cc, 0, 0));
        p[s].A = KEEP(fill(d.a_kind ? (size_t)d.n_heads : (size_t)d.n_heads * d.d_state, 0, 1));
        p[s].D = KEEP(fill(d.d_kind ? d.n_heads : d.d_inner, 0, 0));
        p[s].dt_bias = (d.dt_softplus && id % 2) ? KEEP(fill(d.n_heads, 0, 0)) : NULL;
    }
    orc_inputs in[2];
    for (int s = 0; s < 2; s++) {
        in[s].x = KEEP(fill(tokens * d.d_inner, 0, 0));
        in[s].z = KEEP(fill(tokens * d.d_inner, 0, 0));
        in[s].dt = KEEP(fill(tokens * d.n_heads, !d.dt_softplus, 0));
        in[s].B = KEEP(fill(tokens * GN, 0, 0));
        in[s].C = KEEP(fill(tokens * GN, 0, 0));
    }
    int sel[3] = {d.d_inner - 1, 0, d.d_inner / 2};
    const int n_sel = use_sel ? (d.d_inner >= 3 ? 3 : 1) : 0;
    const size_t width = (size_t)(use_sel ? n_sel : d.d_inner) * (d.combine ? 2 : 1);
    double *out = (double *)malloc((tokens * width + 1) * sizeof(double));
    int rc = orc_bimamba_fwd(&d, &p[0], &p[1], &in[0], (id % 2) ? &in[1] : &in[0], use_sel ? sel : NULL, n_sel, out);
    printf("case %d fwd rc %d sum %.17g\n", id, rc, checksum(out, tokens * width));
    if (with_state) {
        const size_t hs = (size_t)d.batch * d.d_inner * d.d_state, ts = (size_t)d.batch * (d.d_conv - 1) * cc;
        double *h_in = (double *)malloc((hs ? hs : 1) * sizeof(double)), *h_out = (double *)malloc((hs ? hs : 1) * sizeof(double));
        double *t_in = (double *)malloc((ts ? ts : 1) * sizeof(double)), *t_out = (double *)malloc((ts ? ts : 1) * sizeof(double));
        for (size_t i = 0; i < hs; i++) h_in[i] = next_value();
        for (size_t i = 0; i < ts; i++) t_in[i] = next_value();
        for (size_t i = 0; i < hs; i++) h_out[i] = 0.0;
        for (size_t i = 0; i < ts; i++) t_out[i] = 0.0;
        rc = orc_bimamba_block_fwd(&d, &p[0], &p[1], &in[0], &in[0], h_in, d.d_conv > 1 ? t_in : NULL, use_sel ? sel : NULL, n_sel,
                                   out, h_out, d.d_conv > 1 ? t_out : NULL);
        printf("case %d block rc %d sum %.17g state %.17g tail %.17g\n", id, rc, checksum(out, tokens * width),
               checksum(h_out, hs), checksum(t_out, ts));
        double *g = (double *)malloc((tokens * d.d_inner + 1) * sizeof(double));
        rc = orc_one_direction(&d, &p[1], &in[1], -1, NULL, NULL, g, h_out);
        printf("case %d reverse rc %d sum %.17g state %.17g\n", id, rc, checksum(g, tokens * d.d_inner), checksum(h_out, hs));
        free(g); free(h_in); free(h_out); free(t_in); free(t_out);
    }
    free(out);
    for (int i = 0; i < n_owned; i++) free(owned[i]);
    return 0;
}

int main(void)
{
    /*            batch L  Dn  N  H  G  K  a  d  sp bc comb */
    orc_desc cases[] = {
        {1, 1, 1, 4, 1, 1, 1, 0, 0, 0, 0, 0},
        {2, 0, 6, 4, 6, 1, 4, 0, 0, 0, 0, 0},
        {2, 3, 6, 4, 6, 1, 4, 0, 0, 1, 0, 1},
        {1, 2, 8, 16, 2, 1, 4, 1, 1, 1, 1, 0},
        {3, 9, 12, 8, 4, 2, 3, 1, 0, 0, 1, 1},
        {1, 17, 5, 16, 5, 1, 2, 0, 0, 1, 0, 0},
        {2, 5, 128, 4, 4, 4, 4, 0, 1, 0, 1, 0},
    };
    const int n = (int)(sizeof(cases) / sizeof(cases[0]));
    for (int i = 0; i < n; i++) run_case(i, cases[i], i % 2, 1);
    return 0;
}
