/*
 * bimamba.h -- C ABI of the MI355X (gfx950) bidirectional Mamba mixer path.
 *
 * What the library computes (paper Sec. 3.2, eqs. 4-6, and the block variant of Sec. 4.3), per
 * batch element b, direction s in {f (left-to-right), b (right-to-left)}, channel d
 * (head h = d / (d_inner/n_heads), B/C group g = h / (n_heads/n_groups)):
 *
 *   xc_s[t,d] = SiLU(conv_b_s[d] + sum_k conv_w_s[d,k] * x_s[t -/+ (K-1-k), d])      short depthwise conv; causal for f,
 *                                                                                  anti-causal for b; zero outside [0,L)
 *   Delta[t,h] = dt_s[t,h]                       (dt_softplus = 0)
 *              = softplus(dt_s[t,h] + dt_bias_s[h])                (dt_softplus = 1)
 *   h_t[n]    = exp(Delta[t,h] * A_s[h,n]) * h_prev[n] + Delta[t,h] * B_s[t,g,n] * xc_s[t,d]     eq. 4 (t = 0..L-1) / eq. 5 (t = L-1..0)
 *   y_s[t,d]  = sum_n C_s[t,g,n] * h_t[n] + D_s[d] * xc_s[t,d]
 *   g_s[t,d]  = y_s[t,d] * SiLU(z_s[t,d])
 *   out[t,d]  = g_f[t,d] + g_b[t,d]                                                 (BIMAMBA_COMBINE_ADD)
 *   out[t,:]  = [g_f[t,:] | g_b[t,:]]                                               (BIMAMBA_COMBINE_SEPARATE, width 2*d_inner)
 *
 * Eq. 6 adds the two layers' outputs, i.e. after each direction's own output projection.  COMBINE_ADD is that sum only
 * when both directions share one output projection; with untied projections (the paper's setting) use COMBINE_SEPARATE
 * and multiply [g_f | g_b] by the two projection matrices stacked, which realises eq. 6 exactly.
 *
 * With conv_bc = 1 (the Mamba-2 form) B and C pass through the same conv + SiLU as x, using rows
 * d_inner .. d_inner+2*n_groups*d_state-1 of conv_w / conv_b (channel order x | B | C).
 *
 * Memory: every pointer is device memory owned by the caller unless marked "host".  The library allocates nothing and
 * keeps no pointer after a call returns.  What it does keep, per process: per-device caches of launch geometry (the
 * device's CU count, and per kernel variant its occupancy and static LDS), filled the first time a variant is launched
 * on a device, when the library also queries that kernel's attributes and raises its dynamic-LDS limit; the one-shot
 * event pair of bimamba_profile_next_call (per host thread); and the fixed scratch buffer of
 * bimamba_block_fwd_static.  The first-use queries enqueue nothing and are safe under stream capture (a test captures
 * a variant's very first launch).  Activations are token-major with the channel dimension contiguous; batch and token
 * strides are given in elements.
 *
 * Arithmetic: state, decay factors, gate and the sum of eq. 6 are fp32; bf16 I/O is widened on load and rounded
 * to nearest-even once at the final store.  Two kernel families implement the same formulas:
 *   - lane-per-chain kernels (every descriptor): one (direction, batch, channel) recurrence per lane group, all
 *     products and sums in fp32.  When a head's A[h, 0..N-1] is an arithmetic progression in n (checked on the
 *     device, bf16 I/O, d_state <= 32) the N decay factors of a token are formed as a_0 * r^n by repeated
 *     multiplication from two exponentials instead of N exponentials.
 *   - chunked matrix-core kernels (a_kind = SCALAR_PER_HEAD, bf16 I/O, d_state 64 or 128, 32 or 64 channels per
 *     head, time_chunks = state_split = 0): the recurrence over 64-token chunks as dense products on the MFMA
 *     units; their operands (conv output, B, C, the decayed score tile, a copy of the state) are rounded to bf16,
 *     accumulation and the carried state stay fp32.  They read x two channels at a time and the carried state four
 *     states at a time: setting time_chunks or state_split, or passing an x whose pointer is not 4-byte aligned or
 *     whose strides are odd, or an h_in / h_out that is not 16-byte aligned, selects the lane-per-chain kernels for
 *     the call; the workspace size covers both.  A call with few (batch, head) pairs cuts the sequence into time
 *     parts that run concurrently (see bimamba_time_chunks), unless x has a token stride beyond 2^24 elements.
 *
 * Execution: calls validate their arguments on the host, enqueue kernels on the caller's HIP stream
 * and return without synchronising.  Calls on different streams are independent as long as their
 * workspaces do not overlap.
 *
 * Errors: every entry point returns BIMAMBA_OK (0) or a negative bimamba_status.  All codes except
 * BIMAMBA_ERR_HIP are decided on the host before anything is launched.  Nothing throws or aborts.
 */
#ifndef BIMAMBA_H
#define BIMAMBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BIMAMBA_VERSION 1

enum bimamba_status {
    BIMAMBA_OK = 0,
    BIMAMBA_ERR_NULL_POINTER = -1,        /* a required pointer is NULL */
    BIMAMBA_ERR_BAD_SHAPE = -2,           /* non-positive or inconsistent dimension, stride smaller than the row */
    BIMAMBA_ERR_UNSUPPORTED = -3,         /* dtype / d_state / d_conv / grouping / token stride outside the compiled set */
    BIMAMBA_ERR_MISALIGNED = -4,          /* pointer not aligned to its element size (or 16 bytes for the workspace) */
    BIMAMBA_ERR_WORKSPACE_TOO_SMALL = -5, /* workspace_bytes < bimamba_workspace_bytes() */
    BIMAMBA_ERR_HIP = -6,                 /* a launch of this call failed (errors pending from earlier, unrelated calls are
                                             neither reported nor cleared) */
    BIMAMBA_ERR_SCRATCH_EXCEEDED = -7,    /* bimamba_block_fwd_static: the call needs more than BIMAMBA_STATIC_SCRATCH_BYTES */
    BIMAMBA_ERR_ALIAS = -8                /* out may overlap an input view; bimamba_bwd: dpf == dpb (checked on the host) */
};

enum bimamba_dtype { BIMAMBA_F32 = 0, BIMAMBA_BF16 = 1 };
enum bimamba_a_kind {
    BIMAMBA_A_PER_HEAD_STATE = 0,  /* A[n_heads, d_state]; the selective-scan layout has n_heads = d_inner */
    BIMAMBA_A_SCALAR_PER_HEAD = 1  /* A[n_heads]: one decay rate per head (the Mamba-2 form) */
};
enum bimamba_d_kind { BIMAMBA_D_PER_CHANNEL = 0, BIMAMBA_D_PER_HEAD = 1 };
enum bimamba_combine { BIMAMBA_COMBINE_ADD = 0, BIMAMBA_COMBINE_SEPARATE = 1 };

/* Host struct.  Supported: d_state in {4, 8, 16, 32, 64, 128}; 1 <= d_conv <= 4; d_inner % n_heads == 0;
 * n_heads % n_groups == 0; with n_groups > 1, d_inner / n_groups must be a multiple of 64. */
typedef struct bimamba_desc {
    uint32_t struct_size;   /* sizeof(bimamba_desc), checked */
    int32_t batch;          /* >= 0 (0 is a no-op) */
    int32_t seqlen;         /* L >= 0; for bimamba_block_fwd the block length */
    int32_t d_inner;
    int32_t d_state;        /* N */
    int32_t n_heads;        /* H; dt has H channels */
    int32_t n_groups;       /* G; B and C have G*N channels */
    int32_t d_conv;         /* K */
    int32_t io_dtype;       /* bimamba_dtype of x, z, dt, B, C, out, tail_in, tail_out */
    int32_t a_kind;         /* bimamba_a_kind */
    int32_t d_kind;         /* bimamba_d_kind */
    int32_t dt_softplus;    /* 0 or 1 */
    int32_t conv_bc;        /* 0 or 1 */
    int32_t combine;        /* bimamba_combine */
    int32_t time_chunks;    /* 0 = let the library choose; n >= 1 forces the lane-per-chain kernels with n time segments
                               per sequence (segments are scanned in parallel and stitched by a carry pass) */
    int32_t state_split;    /* 0 = let the library choose; 1, 2 or 4 forces the lane-per-chain kernels with that many lanes
                               per (direction, channel) chain, each holding d_state / state_split states (2 needs
                               d_state 16 or 32, 4 needs d_state >= 16); results differ only by the summation order of
                               C_t . h_t */
} bimamba_desc;

/* Per-direction parameters, device pointers, fp32, contiguous.
 * conv_w [conv_ch, d_conv] with conv_ch = d_inner (+ 2*n_groups*d_state if conv_bc); tap d_conv-1 multiplies the
 * current token.  conv_b [conv_ch] or NULL (= 0).  A [n_heads, d_state] or [n_heads].  D [d_inner] or [n_heads].
 * dt_bias [n_heads] or NULL (= 0), read only when dt_softplus = 1. */
typedef struct bimamba_params {
    const float* conv_w;
    const float* conv_b;
    const float* A;
    const float* D;
    const float* dt_bias;
} bimamba_params;

/* One activation tensor [batch, L, channels]: element (b, t, c) lives at ptr + b*stride_batch + t*stride_token + c
 * (in elements of io_dtype).  channels <= stride_token <= 2^26 (BIMAMBA_ERR_UNSUPPORTED beyond: the kernels form row
 * offsets inside a tile of tokens in 32 bits).  Strided views let x, z, dt, B, C be column slices of one projection
 * output.  ptr may be NULL only when batch == 0 or seqlen == 0 (nothing is accessed). */
typedef struct bimamba_tensor {
    void* ptr;
    int64_t stride_batch;
    int64_t stride_token;
} bimamba_tensor;

/* The activations one direction reads: x, z [batch, L, d_inner]; dt [batch, L, n_heads]; B, C [batch, L, n_groups*d_state]. */
typedef struct bimamba_inputs {
    bimamba_tensor x, z, dt, B, C;
} bimamba_inputs;

/*
 * Full-sequence bidirectional mixer path (eqs. 4-6).
 *   desc        host.  pf, pb: host structs of device pointers; pb may equal pf (tied weights).
 *   in_f, in_b  host structs; in_b == NULL or in_b == in_f means both directions read the same activations.
 *   out         [batch, L, d_inner] (ADD) or [batch, L, 2*d_inner] (SEPARATE), io_dtype.  It must not overlap any input
 *               view (BIMAMBA_ERR_ALIAS): byte ranges apart, or, inside one buffer, the same strides (batch stride a
 *               multiple of the token stride) and column ranges apart modulo the token stride.
 *   workspace   device scratch of at least bimamba_workspace_bytes(desc, 0) bytes, 16-byte aligned (may be NULL if 0).
 *   hip_stream  a hipStream_t (NULL = the default stream).
 */
int bimamba_fwd(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                const bimamba_inputs* in_f, const bimamba_inputs* in_b, const bimamba_tensor* out,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Block variant (Sec. 4.3: the forward state is carried across blocks, right-to-left updates stay inside the
 * block).  desc->seqlen is the block length.  The forward scan starts from h_in and its causal conv sees tail_in
 * to the left of the block; the reverse scan starts from zero at the block's right edge with zeros beyond it.
 *   h_in      fp32 [batch, d_inner, d_state] or NULL (= zero state).
 *   tail_in   io_dtype [batch, d_conv-1, tail_ch], the raw (pre-conv) tokens preceding the block, oldest first, or
 *             NULL (= zeros); tail_ch = d_inner (+ 2*n_groups*d_state if conv_bc, channel order x | B | C).
 *   h_out     fp32 [batch, d_inner, d_state]: forward state after the block's last token, or NULL = do not commit.
 *             May alias h_in.
 *   tail_out  io_dtype, same shape as tail_in: last d_conv-1 raw tokens of (tail_in || block), or NULL.  May alias tail_in.
 * A denoising loop calls this once per step with h_out = tail_out = NULL and commits on the block's last step.
 * Everything else as bimamba_fwd; workspace size is bimamba_workspace_bytes(desc, 1).
 */
int bimamba_block_fwd(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                      const bimamba_inputs* in_f, const bimamba_inputs* in_b,
                      const float* h_in, const void* tail_in, float* h_out, void* tail_out,
                      const bimamba_tensor* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * bimamba_block_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results, but
 * the scratch is a fixed buffer of BIMAMBA_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU,
 * held until the process ends); the call allocates and frees nothing.  A descriptor whose
 * bimamba_workspace_bytes(desc, 1) exceeds that size is rejected with BIMAMBA_ERR_SCRATCH_EXCEEDED before anything
 * is launched (batch 16, d_inner 4096 fits blocks of up to 128 tokens in either layout).  All calls on one GPU share
 * the buffer, whatever their stream: two such calls that may overlap in time on the same GPU race; order them on one
 * stream or with events.  Nothing in the buffer has to survive from one call to the next, and nothing in it has to be
 * cleared: every call writes what it reads.
 */
#define BIMAMBA_STATIC_SCRATCH_BYTES (64u << 20)
int bimamba_block_fwd_static(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                             const bimamba_inputs* in_f, const bimamba_inputs* in_b,
                             const float* h_in, const void* tail_in, float* h_out, void* tail_out,
                             const bimamba_tensor* out, void* hip_stream);

/* Gradients with respect to the activations one direction read.  dx, dz [batch, L, d_inner] and ddt [batch, L, n_heads]
 * are views in io_dtype like the inputs (written, one rounding each); dB, dC are contiguous fp32
 * [batch, L, n_groups, d_state] device arrays (sums over the channels of a group, formed in fp32 in a fixed order;
 * overwritten, not accumulated into). */
typedef struct bimamba_input_grads {
    bimamba_tensor dx, dz, ddt;
    float* dB;
    float* dC;
} bimamba_input_grads;

/* Gradients with respect to one direction's parameters: device pointers, fp32, contiguous, shaped like bimamba_params;
 * sums over batch and tokens, zeroed by the library first; the sum over the batch is formed with fp32 atomics, so
 * its last bits can differ between two calls with batch > 2.  dconv_b / ddt_bias may be NULL (not wanted). */
typedef struct bimamba_param_grads {
    float* dconv_w;
    float* dconv_b;
    float* dA;
    float* dD;
    float* ddt_bias;
} bimamba_param_grads;

/*
 * Gradients of bimamba_fwd (the paper trains the model, App. A.2; the backward rule is the chain rule of eqs. 4-6 in
 * the selective form, stated in csrc/bwd_kernels.h).
 *   desc, pf, pb, in_f, in_b   as for bimamba_fwd (in_b == NULL or == in_f: both directions read the same activations).
 *   dout        gradient of bimamba_fwd's out: [batch, L, d_inner] (ADD) or [batch, L, 2*d_inner] (SEPARATE), io_dtype.
 *   din_f       gradients w.r.t. in_f; with shared activations they hold the sum of both directions' contributions
 *               and din_b must be NULL.  With separate activations din_b is required.
 *   dpf, dpb    gradients w.r.t. pf and pb.  If pb == pf (tied weights) the caller adds dpb to dpf; the two must still
 *               be distinct buffers.
 *   workspace   at least bimamba_bwd_workspace_bytes(desc) bytes, 16-byte aligned.
 * Supported: the selective-scan layout, i.e. n_heads == d_inner (Delta, A, D per channel), a_kind PER_HEAD_STATE,
 * d_kind PER_CHANNEL, conv_bc 0, d_state 4, 8 or 16; every other descriptor returns BIMAMBA_ERR_UNSUPPORTED.
 * Nothing may overlap: the gradient views among themselves, the inputs, dout.  (Not checked.)
 * The call enqueues kernels only (its accumulation targets are cleared by a fill kernel, not a memset node) and asks
 * the runtime nothing at first use, so it can be captured into a HIP graph as it is.
 */
int bimamba_bwd(const bimamba_desc* desc, const bimamba_params* pf, const bimamba_params* pb,
                const bimamba_inputs* in_f, const bimamba_inputs* in_b, const bimamba_tensor* dout,
                const bimamba_input_grads* din_f, const bimamba_input_grads* din_b,
                const bimamba_param_grads* dpf, const bimamba_param_grads* dpb,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Workspace of bimamba_bwd: fp32 B|C rows, the state entering every chunk of tokens for both directions
 * (2 * batch * ceil(L / chunk) * d_inner * d_state floats; chunk = 8 tokens, 16 for d_state 4, while the
 * call has at most as many waves as the device has SIMDs; beyond that 8 tokens, 4 for d_state 16), 12 bytes per (batch, token, channel) for the
 * values one direction leaves for the other to add, and the per-wave partial sums of dB and dC. */
size_t bimamba_bwd_workspace_bytes(const bimamba_desc* desc);

/* Bytes of device scratch the two calls above need for this descriptor (0 on an invalid descriptor).  Pure host code. */
size_t bimamba_workspace_bytes(const bimamba_desc* desc, int block_variant);

/* Number of pieces the library would cut the time axis into for this descriptor, each piece scanned by its own
 * workgroups and joined through a carry pass (>= 1; 0 on an invalid descriptor): the time segments of the
 * lane-per-chain kernels, or the time parts of the chunked matrix-core kernels, which are 1 unless a call has so
 * few (batch, head) pairs that they would leave half of the chip empty.  Pure host code. */
int bimamba_time_chunks(const bimamba_desc* desc);

/* Benchmark diagnostics: arm a one-shot probe on the calling host thread.  The next bimamba_fwd or
 * bimamba_block_fwd made by this thread records ev_start immediately before and ev_stop immediately after its
 * scan-and-combine kernel (on the chunked matrix-core path: around its two launches, one per direction; never the
 * B|C preparation, segment summary or tail kernels) on that call's stream, then disarms.  Both are hipEvent_t created by the caller with timing enabled; NULL, NULL disarms.  This thread-local
 * pair is the only state the library keeps between calls. */
void bimamba_profile_next_call(void* ev_start, void* ev_stop);

/* Static, NUL-terminated description of a status code. */
const char* bimamba_status_string(int status);

/* BIMAMBA_VERSION the library was built from. */
int bimamba_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BIMAMBA_H */
