/*
 * rib_attn.h -- C ABI of the RIB window-attention library for AMD MI355X (gfx950).
 *
 * The operator (paper Sec. 2.2 "window-based self-attention"; Sec. 3.1 Eq. 5
 * "concat + scale" and Eq. 6 "score identity"):
 *
 *   A channel-last token grid [B][H][W][C], C = heads*d, channel c = head*d + t,
 *   is cut into (H/M)*(W/M) windows of M x M tokens after a cyclic shift by s:
 *   token n = iy*M + ix (row-major) of window (wy, wx) is the grid pixel
 *       ((wy*M + iy + s) mod H, (wx*M + ix + s) mod W).
 *   Pixels that wrap around attend freely (no mask).  For every image, window
 *   and head, with the N = M*M tokens of the window:
 *
 *       Q_aug[i] = [ scale_c * q[i]  ||  scale_p * f_q[head][i] ]     (Eq. 5)
 *       K_aug[j] = [           k[j]  ||            f_k[head][j] ]
 *       S[i][j]  = < Q_aug[i], K_aug[j] >
 *                = scale_c * q[i].k[j] + scale_p * f_q[i].f_k[j]       (Eq. 6)
 *       P        = softmax over j of S,      O[i] = sum_j P[i][j] v[j]
 *       LSE[i]   = log sum_j exp(S[i][j])    (natural log of the scaled logits)
 *
 *   f_q, f_k are the rank-r positional features of RIB; they depend only on the
 *   position inside the window (Sec. 3.1, last paragraph), so one [heads][N][r]
 *   table serves every window of every image.  The paper's own scales are
 *   scale_c = 1/sqrt(d), scale_p = 1/sqrt(r); any pair may be passed.
 *   S and P are never written to memory and Q_aug / K_aug exist only in
 *   registers and LDS.  O is returned in ORIGINAL grid coordinates.
 *
 * The backward pass is the chain rule through the lines above for a given
 * upstream gradient dO (the paper trains through the operator, Sec. 4 Table 1,
 * without printing it):
 *       dV[j] = sum_i P[i][j] dO[i]          dP[i][j] = dO[i].v[j]
 *       delta_i = dO[i].O[i]                 dS[i][j] = P[i][j] (dP[i][j] - delta_i)
 *       dQ[i] = scale_c sum_j dS[i][j] k[j]  dK[j] = scale_c sum_i dS[i][j] q[i]
 *       dF_q[head][i] = scale_p sum_{images, windows} sum_j dS[i][j] f_k[head][j]
 *       dF_k[head][j] = scale_p sum_{images, windows} sum_i dS[i][j] f_q[head][i]
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller, valid on the
 *     current HIP device, and at least 4-byte aligned (the kernels move bf16
 *     values in pairs; 16-byte alignment, as allocators give, is the fast case).
 *     A misaligned pointer is rejected with RIB_ERR_SHAPE.  Unless an entry point says otherwise the library
 *     allocates nothing, frees nothing and keeps no pointer after returning.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work
 *     is enqueued asynchronously; nothing synchronises.
 *   - Arguments are validated on the host BEFORE anything is launched; a failed
 *     validation returns an error code and touches no memory.  No C++ exception
 *     crosses the boundary.
 *   - Outputs must not overlap inputs or each other.
 *   - Entry points are thread-safe.  The only state the library keeps is a record, per
 *     device, of one-time set-up (a kernel's dynamic-LDS limit raised, the number
 *     of compute units, the address of the static scratch below); a failed
 *     set-up is not remembered and is tried again by the next call.
 */
#ifndef RIB_ATTN_H
#define RIB_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RIB_OK = 0,
    RIB_ERR_NULL = 1,        /* a required pointer is NULL */
    RIB_ERR_SHAPE = 2,       /* non-positive size, H or W not a multiple of window, shift out of range, bad stride,
                                unknown flag bit, data pointer not 4-byte aligned */
    RIB_ERR_DTYPE = 3,       /* dtype is not one of rib_dtype */
    RIB_ERR_UNSUPPORTED = 4, /* valid problem, but d / r beyond what the kernels are built for */
    RIB_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or smaller than rib_window_attn_bwd_workspace_bytes */
    RIB_ERR_LAUNCH = 6       /* HIP reported an error when a kernel was enqueued.  The library reads (and thereby
                                clears) the calling thread's last HIP error after each launch, so an error that
                                an earlier HIP call of the caller left pending is reported here as well */
} rib_status;

typedef enum {
    RIB_F32 = 0,             /* fp32 storage, fp32 arithmetic */
    RIB_BF16 = 1             /* bf16 storage, bf16 matrix-core operands, fp32 accumulation and softmax state */
} rib_dtype;

/* Flags for rib_params.flags. */
enum {
    /* Always track the running row maximum in the online softmax.  By default the
     * matrix-core forward first runs without it and checks every row's
     * denominator against a safe range afterwards, redoing a workgroup with max
     * tracking only if a row fails.  Results are the same within rounding; this
     * exists so that both code paths can be tested and timed. */
    RIB_FLAG_FORCE_ROW_MAX = 1,
    /* Use the wide workgroups (8 waves sharing each streamed tile) whenever the
     * window has a multiple of 512 tokens, forward and backward.  By default
     * they are chosen only for windows of 4096 tokens or more with enough work
     * to fill the chip several times over.  Same results within rounding (tile
     * boundaries do not enter the arithmetic).  For tests and tuning. */
    RIB_FLAG_WIDE = 2,
    /* Run on the vector-ALU kernels even where a matrix-core kernel serves the
     * problem.  Same results within rounding; for tests and comparisons. */
    RIB_FLAG_VECTOR_ONLY = 4
};

typedef struct {
    int32_t B, H, W;         /* grid: images, rows, columns */
    int32_t heads, d, r;     /* heads, head dim, RIB rank (r may be 0: plain window attention) */
    int32_t window;          /* M; H % M == 0 and W % M == 0 are required (pad upstream) */
    int32_t shift;           /* s; 0 <= s < M */
    float scale_c, scale_p;  /* logit scales of the content and positional parts (Eq. 5) */
    int32_t dtype;           /* rib_dtype of q, k, v, f_q, f_k, out, d_out, dq, dk, dv */
    int32_t flags;           /* RIB_FLAG_* */
    int64_t token_stride;    /* elements between consecutive tokens of q, k and v; 0 means dense (= C).
                                Lets q, k, v be views into one packed [B][H][W][3C] projection. */
} rib_params;

/* Built for: 1 <= d <= 64, 0 <= r <= 64, any window side M with M*M <= 65536.
 * Problems with d <= 32 and d + r <= 64 run on the matrix-core kernels (bf16
 * storage: bf16 MFMA with fp32 accumulation; fp32 storage: fp32 MFMA);
 * everything else runs on a slower fp32 vector-ALU kernel with the same results. */

/* Forward:  out[B][H][W][C]  (dtype of q),  lse[B*nW][heads][N] fp32 or NULL.
 *   q, k, v : [B][H][W] tokens of C channels, token stride p->token_stride
 *   f_q,f_k : [heads][N][r], dense; may be NULL iff r == 0
 *   lse     : window index w = (b*(H/M) + wy)*(W/M) + wx; pass NULL for inference
 * Returns RIB_OK once the kernels are enqueued on `stream`. */
rib_status rib_window_attn_fwd(const rib_params *p,
                               const void *q, const void *k, const void *v,
                               const void *f_q, const void *f_k,
                               void *out, float *lse, void *stream);

/* Bytes of device scratch rib_window_attn_bwd needs for this problem (0 if the
 * parameters are invalid).  The caller allocates it, 256-byte aligned. */
size_t rib_window_attn_bwd_workspace_bytes(const rib_params *p);

/* Backward.  `out` and `lse` are the results of rib_window_attn_fwd on the same
 * inputs.  dq, dk, dv [B][H][W][C] (dense, dtype of q) and df_q, df_k
 * [heads][N][r] fp32 are OVERWRITTEN (df_* are sums over all images and
 * windows, reduced in a fixed order: results are run-to-run identical).
 * df_q / df_k may be NULL iff r == 0.  `workspace` is scratch for the duration
 * of the enqueued work; its contents afterwards are unspecified. */
rib_status rib_window_attn_bwd(const rib_params *p,
                               const void *q, const void *k, const void *v,
                               const void *f_q, const void *f_k,
                               const void *out, const void *d_out, const float *lse,
                               void *dq, void *dk, void *dv,
                               float *df_q, float *df_k,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Size of the library's own backward scratch (see below): a static device array of
 * this many bytes, which every GPU the library is loaded on holds until the process
 * ends. */
#define RIB_STATIC_SCRATCH_BYTES (32u << 20)

/* rib_window_attn_bwd for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP graph capture, tight serving / training loops,
 * harnesses that forbid hipMalloc.  Same arguments, results (bit for bit) and
 * errors as rib_window_attn_bwd, but the scratch is a static device array inside
 * the library; the call allocates nothing, frees nothing and calls no allocating
 * routine.  Problems whose rib_window_attn_bwd_workspace_bytes exceed
 * RIB_STATIC_SCRATCH_BYTES are rejected with RIB_ERR_WORKSPACE before anything is
 * launched.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on the same GPU (different streams or threads) race on it; calls on one
 * stream, or otherwise ordered, are safe.  Nothing in the array has to start at
 * zero and nothing is kept in it between calls. */
rib_status rib_window_attn_bwd_static_scratch(const rib_params *p,
                                              const void *q, const void *k, const void *v,
                                              const void *f_q, const void *f_k,
                                              const void *out, const void *d_out, const float *lse,
                                              void *dq, void *dk, void *dv,
                                              float *df_q, float *df_k, void *stream);

/* ------------------------------------------------------------------------
 * Gated variants: the convolutional-local-attention gate of the paper's Sec. 3.2
 * Eq. 9, O' = O (.) G, applied in the attention kernel's epilogue instead of in
 * a separate elementwise pass (the convolutions and the sigmoid that produce G,
 * Eq. 8, stay with the caller).  `gate` is a dense [B][H][W][C] tensor in the
 * problem's storage type, in ORIGINAL grid coordinates like q, k, v.
 *
 * Forward: out_gated = O (.) gate.  out_raw (may be NULL for inference) receives
 * the ungated O, which the backward needs.  Everything else as
 * rib_window_attn_fwd. */
rib_status rib_window_attn_gated_fwd(const rib_params *p,
                                     const void *q, const void *k, const void *v,
                                     const void *f_q, const void *f_k, const void *gate,
                                     void *out_gated, void *out_raw, float *lse, void *stream);

/* Scratch bytes for rib_window_attn_gated_bwd (the plain backward's scratch plus
 * one grid tensor for dO; a multiple of 256, 0 if *p is invalid). */
size_t rib_window_attn_gated_bwd_workspace_bytes(const rib_params *p);

/* Backward of the gated operator from d_out_gated = dL/dO':
 *     dO = dO' (.) G    (formed once, in the storage type, inside the workspace)
 *     dG = dO' (.) O    (written to dgate, [B][H][W][C], storage type)
 * followed by the backward of the plain operator with that dO; one pass over the
 * grid produces dO, dG and delta together.  out_raw is the UNGATED forward
 * output.  Arguments, errors and determinism otherwise as rib_window_attn_bwd. */
rib_status rib_window_attn_gated_bwd(const rib_params *p,
                                     const void *q, const void *k, const void *v,
                                     const void *f_q, const void *f_k, const void *gate,
                                     const void *out_raw, const void *d_out_gated, const float *lse,
                                     void *dq, void *dk, void *dv, void *dgate,
                                     float *df_q, float *df_k,
                                     void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * RIB feature generator (paper Sec. 3.1 Eq. 1-3): produces the f_q, f_k tables
 * the attention entry points above consume.  For an M x M window every token
 * n = iy*M + ix has the coordinate pair x = (-1 + 2 iy/(M-1), -1 + 2 ix/(M-1))
 * (row first; the single token of M = 1 sits at 0), and
 *
 *   r_in = [ x, sin(2^0 x), cos(2^0 x), ..., sin(2^(L-1) x), cos(2^(L-1) x) ]   (Eq. 1, width 2+4L)
 *   h    = ReLU(r_in W_h + b_h)                                                  (Eq. 2, width d_h)
 *   f_q[head] = h W_pq[head],    f_k[head] = h W_pk[head]                        (Eq. 3, width r)
 *
 * h is shared by all heads; the projections are per head and have no bias.
 * The tables depend only on M and the weights, so a caller computes them once
 * per weight update and window size (Sec. 3.1, last paragraph).
 *
 * Layouts (all dense, row-major, DEVICE pointers): W_h [2+4L][d_h], b_h [d_h],
 * W_pq, W_pk [heads][d_h][r] -- always fp32; f_q, f_k [heads][M*M][r] in
 * `dtype` storage (bf16: rounded to nearest even from the fp32 result).
 * Arithmetic: coordinates and their sines / cosines in fp64, rounded once to
 * fp32; the two matrix products in fp32. */
typedef struct rib_gen_params {
    int32_t window;   /* M, 1..256 */
    int32_t heads;    /* 1..64 */
    int32_t r;        /* 1..64 */
    int32_t L;        /* Fourier bands, 0..16 (paper: 10) */
    int32_t d_h;      /* hidden width, 1..64 (paper: 32) */
    int32_t dtype;    /* rib_dtype of f_q, f_k */
} rib_gen_params;

/* Enqueue the generator forward.  Errors: RIB_ERR_NULL, RIB_ERR_SHAPE (a size
 * outside the ranges above), RIB_ERR_DTYPE, RIB_ERR_LAUNCH. */
rib_status rib_features_fwd(const rib_gen_params *p, const float *W_h, const float *b_h,
                            const float *W_pq, const float *W_pk, void *f_q, void *f_k, void *stream);

/* Bytes of scratch rib_features_bwd needs (a multiple of 256; 0 if *p is invalid). */
size_t rib_features_bwd_workspace_bytes(const rib_gen_params *p);

/* Enqueue the generator backward: from df_q, df_k [heads][M*M][r] fp32 (what
 * rib_window_attn_bwd returns, possibly summed over layers that share the
 * generator) to the gradients of the four weight tensors, fp32, same shapes as
 * the weights, OVERWRITTEN.  Chain rule through Eq. 3, 2 (ReLU passes the
 * gradient where its input is positive) and the linear layer of Eq. 2; sums
 * over tokens run in a fixed order (run-to-run identical results).  `workspace`
 * is device scratch, 256-byte aligned, at least
 * rib_features_bwd_workspace_bytes(p) bytes, owned by the caller (else
 * RIB_ERR_WORKSPACE). */
rib_status rib_features_bwd(const rib_gen_params *p, const float *W_h, const float *b_h,
                            const float *W_pq, const float *W_pk, const float *df_q, const float *df_k,
                            float *dW_h, float *db_h, float *dW_pq, float *dW_pk,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Static, NUL-terminated description of a status code. */
const char *rib_status_string(rib_status st);

/* Name of the kernel family that would serve this problem: "mfma-bf16" (bf16
 * storage on the bf16 matrix instructions), "mfma-f32" (fp32 storage on the
 * fp32 matrix instruction) or "valu-f32" (vector ALU, any storage); NULL if the
 * parameters are invalid.  For logs and tests. */
const char *rib_window_attn_kernel_name(const rib_params *p, int backward);

#ifdef __cplusplus
}
#endif
#endif /* RIB_ATTN_H */
