/*
 * ssg -- FP8 SwiGLU MLP block with Smooth-SwiGLU for AMD MI355X (gfx950).
 *
 * C ABI of libssg.so.  The block is the one the paper states in Sections 4.1
 * and 4.4: for token t and channel i
 *
 *     U_ti = x_t . w1_i      (linear branch)        W1 [f,d] row-major, row i = w1_i
 *     G_ti = x_t . w2_i      (Swish branch)         W2 [f,d]
 *     h_ti = U_ti * G_ti * sigma(G_ti)
 *     y_t  = sum_i w3_i h_ti (last linear layer)    W3 [d,f] row-major, column i = w3_i
 *
 * with every matrix product done on FP8 operands (E4M3 for activations and
 * weights, E5M2 for gradients, Section 2 and 6.2) and fp32 accumulation.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned,
 *     row-major with the last index contiguous.  The library never allocates
 *     device memory and keeps no state between calls.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work and return; nothing is synchronised.
 *   - Errors: SSG_ERR_ARG, SSG_ERR_SHAPE, SSG_ERR_WORKSPACE and SSG_ERR_UNSUPPORTED
 *     are found before anything is enqueued (every argument, buffer size and
 *     internal launch configuration is checked first), and so is a HIP error that
 *     was already pending when the call was made (SSG_ERR_HIP, nothing launched;
 *     the pending error is consumed).  SSG_ERR_HIP after that means one of the
 *     call's own launches failed: the outputs are then undefined.
 *     ssg_last_error() returns a description (thread-local, valid until the next
 *     call on that thread).
 *   - Buffers whose size the library computes (`saved`, `workspace`, `prepared`)
 *     are passed with their size in bytes; a buffer smaller than the matching
 *     *_bytes() query returns SSG_ERR_WORKSPACE.
 *   - Matrix extents that are contracted or vector-accessed (every rows/cols,
 *     T, d, f, M, N, K below) must be positive multiples of 16, otherwise
 *     SSG_ERR_SHAPE; ssg_amax / ssg_quantize accept an extent of 0 as "nothing
 *     to do" (amax = 0, scale = 1).
 *   - Inputs are expected to be finite.  NaN is ignored by every amax and maps
 *     to the format's NaN code with its sign; +-Inf saturates like any value
 *     above the largest finite one.
 */
#ifndef SSG_H
#define SSG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SSG_OK = 0,
    SSG_ERR_ARG = -1,          /* null pointer, bad enum, misaligned pointer */
    SSG_ERR_SHAPE = -2,        /* extent not a positive multiple of 16, or too large */
    SSG_ERR_WORKSPACE = -3,    /* a caller-allocated buffer is smaller than its *_bytes() query, or the shape is beyond
                                  what the static scratch of ssg_infer_fwd_noalloc holds */
    SSG_ERR_HIP = -4,          /* a launch reported an error (text in ssg_last_error) */
    SSG_ERR_UNSUPPORTED = -5
} ssg_status;

typedef enum { SSG_E4M3 = 0, SSG_E5M2 = 1 } ssg_fp8_format;      /* OCP FP8 encodings (Section 2) */
typedef enum { SSG_BF16 = 0, SSG_F32 = 1 } ssg_dtype;
typedef enum { SSG_SCALE_CURRENT = 0,   /* scale from this tensor's own range ("just-in-time", Section 2) */
               SSG_SCALE_GIVEN = 1,     /* caller supplies the scale, e.g. from earlier iterations ("delayed") */
               SSG_SCALE_DELAYED = 2    /* ssg_mlp_desc only: scales come from the amax history in `scaling_state` */
} ssg_scale_mode;
typedef enum { SSG_ROUND_EXACT_DIV = 0, /* scale = fl32(fmax / amax) */
               SSG_ROUND_POW2 = 1       /* scale = 2^floor(log2(fmax / amax)) */
} ssg_scale_round;

const char *ssg_last_error(void);
const char *ssg_version(void);

/* Largest absolute value of a tensor of n elements (per-tensor range, Section 2).
 * amax_dev: out, one float.  NaN elements are ignored. */
ssg_status ssg_amax(const void *src, ssg_dtype src_dtype, size_t n, float *amax_dev, void *stream);

/* The quantization function Q of Eq. 2 for one tensor [rows, cols]:
 *     dst[r,c] = satcast_fmt( fl32( src[r,c] * scale ) )
 * satcast = round to nearest even, subnormals kept, magnitudes above the
 * largest finite value clamp to it.  CURRENT: scale = fl32(fmax/amax) (1 when
 * amax = 0, largest finite float when the division overflows), written to
 * *scale_dev; GIVEN: *scale_dev is read.
 *   dst     out [rows, cols] bytes
 *   dst_t   out [cols, rows] bytes, the transposed copy (may be NULL)
 *   amax_dev out, one float; required for CURRENT (holds the amax afterwards),
 *           may be NULL for GIVEN */
ssg_status ssg_quantize(const void *src, ssg_dtype src_dtype, int64_t rows, int64_t cols,
                        ssg_fp8_format fmt, ssg_scale_mode mode, ssg_scale_round rnd,
                        uint8_t *dst, uint8_t *dst_t, float *scale_dev, float *amax_dev, void *stream);

/* One FP8 contraction with fp32 accumulation (the matrix products of Eq. 2 and
 * of the display that follows it):
 *     C[m,n] = ( sum_k A[m,k] * B[n,k] ) / (sa * sb)
 * A [M,K] codes of a_fmt, B [N,K] codes of b_fmt (b_fmt must be SSG_E4M3),
 * C [M,N] of c_dtype.  sa_dev / sb_dev: device pointers to the operands'
 * scales (NULL = 1). */
ssg_status ssg_gemm_fp8(const uint8_t *A, ssg_fp8_format a_fmt, const uint8_t *B, ssg_fp8_format b_fmt,
                        int64_t M, int64_t N, int64_t K, const float *sa_dev, const float *sb_dev,
                        void *C, ssg_dtype c_dtype, void *stream);
/* The same contraction with "K-major" operands: a_kmajor = 1 means A is stored as [K,M] (M contiguous),
 * b_kmajor = 1 that B is stored as [K,N].  This is how the backward contractions read the tensors the
 * forward quantized row-major -- dY^ [T,d], h^ [T,f], x^ [T,d], dU^ [T,f] for the weight gradients (contraction
 * over T), w^ [f,d] and w3~ [d,f] for the input gradients -- without transposed copies.  Built combinations:
 * (0,0), (0,1), (1,1); (1,0) returns SSG_ERR_UNSUPPORTED. */
ssg_status ssg_gemm_fp8_layout(const uint8_t *A, ssg_fp8_format a_fmt, int a_kmajor, const uint8_t *B,
                               ssg_fp8_format b_fmt, int b_kmajor, int64_t M, int64_t N, int64_t K,
                               const float *sa_dev, const float *sb_dev, void *C, ssg_dtype c_dtype, void *stream);

/* SwiGLU product of Section 4.1 from stored bf16 U, G [T,f], in fp32:
 * h = u * (g * (1 / (1 + exp(-g)))).  Debug / test entry: this is the h the
 * fused kernels quantize.  h out [T,f] float. */
ssg_status ssg_swiglu(const void *U, const void *G, int64_t T, int64_t f, float *h, void *stream);

/* Smooth-SwiGLU quantization of the SwiGLU product (Section 4.4, Eq. 2 and the
 * three-step per-channel recipe): from bf16 U, G [T,f]
 *     a_i = max_t |h_ti|,  s_i = fl32(448 / a_i),  sinv_i = fl32(a_i / 448)   (both 1 when a_i = 0)
 *     h_q[t,i] = satcast_E4M3( fl32( h_ti * s_i ) )
 * smooth = 0 gives the plain block of Figure 4(a): one scale for the whole
 * tensor, s_i = fl32(448 / max_i a_i) for every i and sinv_i = 1.
 *   h_q   out [T,f];  h_qT out [f,T] (may be NULL)
 *   s, sinv, camax  out, f floats each (camax = a_i) */
ssg_status ssg_smooth_swiglu_quantize(const void *U, const void *G, int64_t T, int64_t f, int smooth,
                                      uint8_t *h_q, uint8_t *h_qT, float *s, float *sinv, float *camax,
                                      void *stream);

/* Folding the inverse factor into the last linear layer, w3~_i = Q(s_i^-1 * w3_i)
 * (the display after Eq. 2): W3 bf16 [d,f], column i scaled by sinv_i in fp32,
 * then per-tensor E4M3 of the result.
 *   w3_q out [d,f]; w3_qT out [f,d] (may be NULL)
 *   w3_camax out, f floats (max_j |W3_ji|); scale_dev, amax_dev out, one float each */
ssg_status ssg_fold_w3(const void *W3, const float *sinv, int64_t d, int64_t f,
                       uint8_t *w3_q, uint8_t *w3_qT, float *w3_camax, float *scale_dev, float *amax_dev,
                       void *stream);

/* ---- the whole block ---------------------------------------------------- */

typedef struct {
    int64_t T, d, f;
    int32_t smooth;          /* 1 = Smooth-SwiGLU (Figure 4b), 0 = plain per-tensor Q(h) (Figure 4a) */
    int32_t rnd;             /* ssg_scale_round, applied to the per-tensor scales */
    int32_t y_dtype;         /* ssg_dtype of y and dx */
    int32_t dw_dtype;        /* ssg_dtype of dW1, dW2, dW3 */
    int32_t weights_cached;  /* 1 = W1, W2, W3 are unchanged since an earlier ssg_mlp_fwd that used this same `saved`
                                buffer: keep its Q(w1), Q(w2), their scales and W3's per-channel
                                ranges instead of recomputing them (quantize once per optimizer step, run many
                                micro-batches).  0 = quantize the weights in this call. */
    int32_t scale_mode;      /* SSG_SCALE_CURRENT, or SSG_SCALE_DELAYED (needs scaling_state): the per-tensor scales of
                                x, W1, W2, dY, dU, dG come from the ranges of earlier calls (Section 2 "delayed
                                scaling", what the runs of Section 6.2 used), so no stand-alone range pass runs;
                                values beyond the remembered range saturate.  The per-channel factors of
                                Smooth-SwiGLU and the scale of the folded w3 stay current. */
    int32_t h_scale_mode;    /* plain block (smooth = 0) only: SSG_SCALE_CURRENT = the scale of h comes from its own
                                range; SSG_SCALE_GIVEN = *h_scale is used as it is (a scale from earlier iterations,
                                Section 2): values beyond the range it allows saturate (Section 3).  Must be
                                SSG_SCALE_CURRENT when smooth = 1. */
    int32_t keep_bf16_grads; /* SSG_SCALE_DELAYED only (no effect otherwise): 1 = ssg_mlp_bwd also stores the bf16 dU, dG
                                that the fused epilogue rounds and casts from (for inspection; under current scaling
                                they are always stored).  0 = only their E5M2 codes are written. */
    int32_t w3_layer_bf16;   /* 1 = the comparison variant of Section 4.3 / Table 3 ("FP8 + SwiGLU output in BF16"): the
                                quantization of the last linear layer is disabled -- the SwiGLU product is rounded once to
                                bf16 and y = h W3^T, dH = dY W3 and dW3 = dY^T h run on bf16 operands (no scales, no
                                per-channel factors); the other six contractions stay FP8.  Needs smooth = 0 and current
                                scaling.  `saved` and `workspace` are larger (transposed bf16 copies of h, W3 and dY). */
    int32_t reserved[3];     /* must be 0 */
    void *scaling_state;     /* device, ssg_mlp_scaling_state_bytes() bytes, or NULL.  When given, every call
                                (current or delayed) enters the ranges it saw into the history. */
    const float *h_scale;    /* device, one float: the given scale of h (h_scale_mode = SSG_SCALE_GIVEN), else NULL */
    uint64_t *h_counters;    /* device, two 64-bit words, or NULL.  When given, ssg_mlp_fwd clears them and the cast of
                                the SwiGLU product counts into [0] the elements that overflow E4M3 under their scale
                                (scaled magnitude beyond 464 = 448 plus half the spacing of the top binade: only the
                                clamp of the saturating cast keeps them finite) and into [1] the nonzero elements
                                whose code is +-0 (underflow) -- the two failure modes of Section 3. */
} ssg_mlp_desc;

/* Amax history of delayed scaling.  One state per block instance, kept by the caller across steps,
 * initialised once with ssg_mlp_scaling_init (empty history: scale 1).  Reading used (the paper gives
 * none): history of the last 16 calls per tensor, scale = fl32(fmax / largest entry) with the rounding
 * of desc.rnd, margin 0; the range seen in a call replaces the oldest entry after the call.  A first
 * call under SSG_SCALE_CURRENT with the state attached fills the history with real ranges.
 * Layout (32-bit words): tensor k = 0..5 (x, w1, w2, dy, du, dg) owns words [32k, 32k+32):
 * [0] scale the next call uses (float), [1] ring position, [2] range seen in the last call (float),
 * [8..24) the ring of ranges (float).  With weights_cached = 1 the entries of w1, w2 are left alone. */
size_t ssg_mlp_scaling_state_bytes(void);
ssg_status ssg_mlp_scaling_init(void *scaling_state, void *stream);

/* Sizes of the two caller-allocated device buffers.  `saved` carries what the
 * backward pass needs (quantized operands, bf16 U and G, the factors); `workspace` is scratch of the backward pass.  0 on a bad
 * descriptor. */
size_t ssg_mlp_saved_bytes(const ssg_mlp_desc *desc);
size_t ssg_mlp_workspace_bytes(const ssg_mlp_desc *desc);

/* Forward: y = block(x).  x [T,d], W1, W2 [f,d], W3 [d,f] bf16; y [T,d] of y_dtype.
 * saved: out, saved_bytes >= ssg_mlp_saved_bytes(desc), else SSG_ERR_WORKSPACE. */
ssg_status ssg_mlp_fwd(const ssg_mlp_desc *desc, const void *x, const void *W1, const void *W2,
                       const void *W3, void *y, void *saved, size_t saved_bytes, void *stream);

/* Backward of sum(y * dy) with the straight-through estimator through every Q
 * and s_i held constant: dy [T,d] bf16 is quantized to E5M2; dx [T,d] y_dtype;
 * dW1, dW2 [f,d], dW3 [d,f] of dw_dtype.  saved: as the forward call with the same desc left it;
 * workspace: scratch, workspace_bytes >= ssg_mlp_workspace_bytes(desc); either buffer too small:
 * SSG_ERR_WORKSPACE. */
ssg_status ssg_mlp_bwd(const ssg_mlp_desc *desc, const void *dy, const void *saved, size_t saved_bytes, void *dx,
                       void *dW1, void *dW2, void *dW3, void *workspace, size_t workspace_bytes, void *stream);

/* Pointers into `saved` / `workspace` for tests and reports (host struct of device pointers). */
typedef struct {
    const float *scales;     /* [0]=sx [1]=sw1 [2]=sw2 [3]=sw3 [4]=amax_x [5]=amax_w1 [6]=amax_w2 [7]=amax of s^-1*w3
                                [8]=amax of h (plain block only) ([4..6] are written under current scaling only) */
    const float *s, *sinv, *h_camax, *w3_camax;          /* f floats each */
    const uint8_t *x_q, *w1_q, *w2_q, *h_q, *w3_q;       /* [T,d], [f,d], [f,d], [T,f], [d,f]: row-major only; the
                                                            backward reads them K-major, no transposed copies */
    const void *U, *G;                                   /* bf16 [T,f] */
    const void *h_b, *h_bT, *w3T;                        /* w3_layer_bf16 = 1 only (else NULL): bf16 SwiGLU output [T,f],
                                                            its transpose [f,T], W3 transposed [f,d] */
} ssg_mlp_saved_view;
typedef struct {
    const float *scales;     /* [0]=sdy [1]=sdu [2]=sdg [3]=amax_dy [4]=amax_du [5]=amax_dg ([3..5]: current scaling only) */
    const uint8_t *dy_q, *du_q, *dg_q;                   /* [T,d], [T,f], [T,f] */
    const void *dU, *dG;                                 /* bf16 [T,f]; under SSG_SCALE_DELAYED the dH epilogue emits the
                                                            E5M2 codes directly and these are written only when
                                                            desc.keep_bf16_grads = 1 */
    const void *dyT;                                     /* w3_layer_bf16 = 1 only (else NULL): bf16 dY transposed [d,T] */
} ssg_mlp_workspace_view;
/* How ssg_mlp_bwd shares the weight gradient of the last layer (dW3, derived from the display after Eq. 2) between
 * its two grouped GEMM launches on a GPU with `compute_units` compute units: workgroups come in sets of 8 output
 * tiles; *dw3_sets_total receives the number of sets of dW3, *dw3_sets_first how many of them run in the first
 * launch (beside dH), the rest running in the second (beside dX, dW1, dW2).  The choice minimises the predicted
 * time of the two launches; it changes no result.  Host pointers; nothing is launched and no GPU is needed (the
 * call ssg_mlp_bwd makes uses the compute unit count of the current device).  *dw3_sets_first = *dw3_sets_total
 * where the grouped launches are not used (w3_layer_bf16 = 1, shapes whose input gradient takes two launches). */
ssg_status ssg_mlp_bwd_plan(const ssg_mlp_desc *desc, int32_t compute_units, int32_t *dw3_sets_first,
                            int32_t *dw3_sets_total);
ssg_status ssg_mlp_view_saved(const ssg_mlp_desc *desc, const void *saved, ssg_mlp_saved_view *out);
ssg_status ssg_mlp_view_workspace(const ssg_mlp_desc *desc, const void *workspace, ssg_mlp_workspace_view *out);

/* ---- inference with the factors folded into the weights (end of Section 4.4) --------
 * With the per-channel factors fixed (s, sinv: the two f-vectors a calibration call of ssg_mlp_fwd
 * left in its `saved` buffer), they are absorbed once into the weights,
 *     w1~_i = Q(s_i w1_i)     w2^ = Q(w2)     w3~_i = Q(s_i^-1 w3_i)        (per-tensor E4M3 each)
 * and a forward call does no per-channel work: x^ = Q(x); one GEMM kernel forms both inner
 * products, the SwiGLU product (s_i u_i) Swish(g_i) from the dequantized fp32 inner products and
 * casts it to E4M3 as it stands (no bf16 U, G are stored: nothing is kept for a backward pass);
 * y = h^ w3~^T / sigma_w3.
 * desc: the block's T, d, f, rnd, y_dtype (smooth must be 1, scale_mode current; T may differ from call
 * to call with the same `prepared`).  prepared / workspace: device, caller-owned, sizes from the two
 * queries, passed with their sizes in bytes.  W1, W2 [f,d], W3 [d,f], x [T,d] bf16; s, sinv [f] fp32;
 * y [T,d] y_dtype.  Asynchronous, nothing allocated. */
typedef struct {
    const float *weight_scales;   /* [0]=scale of w1~ [1]=scale of w2^ [2]=scale of w3~ [4..6] their ranges */
    const uint8_t *w1_q, *w2_q;   /* [f,d] */
    const uint8_t *w3_q;          /* [d,f] */
    const float *x_scale;         /* [0]=scale of x^ [1]=range of x (last call) */
    const uint8_t *x_q, *h_q;     /* [T,d], [T,f] of the last call */
} ssg_infer_view_t;
size_t ssg_infer_prepared_bytes(const ssg_mlp_desc *desc);
size_t ssg_infer_workspace_bytes(const ssg_mlp_desc *desc);
ssg_status ssg_infer_prepare(const ssg_mlp_desc *desc, const void *W1, const void *W2, const void *W3, const float *s,
                             const float *sinv, void *prepared, size_t prepared_bytes, void *stream);
ssg_status ssg_infer_fwd(const ssg_mlp_desc *desc, const void *x, const void *prepared, size_t prepared_bytes, void *y,
                         void *workspace, size_t workspace_bytes, void *stream);
/* ssg_infer_fwd for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  The workspace of the call
 * (x^ [T,d], h^ [T,f], the range slots of x) lies in a static device array inside the library instead
 * (ssg_infer_noalloc_max_bytes() = 16 MiB, held by every GPU the library runs on until the process ends); a shape
 * with ssg_infer_workspace_bytes(desc) beyond that returns SSG_ERR_WORKSPACE with nothing launched.  Same kernels
 * and same results as ssg_infer_fwd; no hipMalloc, hipFree or allocating library routine is called, and the range
 * slots are cleared by a small fill kernel (no memset node).  All calls on one GPU share that GPU's array, which
 * keeps the last call's contents: calls that overlap in time on one GPU (two streams, two threads) race and must
 * be serialised by the caller.  The array's device address is looked up once per GPU on the first call there. */
size_t ssg_infer_noalloc_max_bytes(void);
ssg_status ssg_infer_fwd_noalloc(const ssg_mlp_desc *desc, const void *x, const void *prepared, size_t prepared_bytes,
                                 void *y, void *stream);
ssg_status ssg_infer_view(const ssg_mlp_desc *desc, const void *prepared, const void *workspace, ssg_infer_view_t *out);

/* ---- Adam with both moments in FP8 (Section 5) -------------------------------
 * The first moment is stored in E4M3 and the second in E5M2 (Section 5.2), each with one
 * per-tensor scale chosen from the range of the new moment as in Section 2
 * (scale = fl32(fmax / amax), code = satcast(fl32(value * scale))).  One step on a flat tensor:
 *     m_prev = fl32(decode(m_q) fl32(1/scale_m))  v_prev = fl32(decode(v_q) fl32(1/scale_v))
 *     m = fl32(fl32(beta1 m_prev) + fl32((1-beta1) g))
 *     v = fl32(fl32(beta2 v_prev) + fl32(fl32((1-beta2) g) g))
 *     upd = fl32(fl32(m c1) / fl32(sqrt(fl32(v c2)) + eps)),  c_i = fl32(1 / (1 - beta_i^step))
 *     w = fl32(w - fl32(lr fl32(upd + fl32(weight_decay w))))           (decoupled decay)
 *     m_q, scale_m = Q_E4M3(m);  v_q, scale_v = Q_E5M2(v)
 * (the update uses the unrounded moments of this step; fl32 = one rounded binary32 operation).
 * The paper fixes the two formats; the rest is this library's reading.
 *
 * state (device, caller-owned, ssg_adam_state_bytes(n) bytes, 256-byte aligned): scale and range
 * words kept twice by step parity, the range slots of the reduction, then m_q[n] and v_q[n].
 * ssg_adam_init writes zero moments (codes 0, scales 1).  ssg_adam_step takes step = 1, 2, 3, ...
 * in order (the parity of `step` selects which scalar set is read and which is written).
 * grad: [n] device, grad_dtype SSG_F32 or SSG_BF16.  w: [n] fp32 device, updated in place.
 * w_bf16: optional [n] bf16 device copy of the new weights (NULL to skip).  n: multiple of 16,
 * below 2^40.  All calls are asynchronous on `stream` and allocate nothing. */
typedef struct {
    int64_t n;
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;            /* >= 1 */
    int32_t grad_dtype;      /* ssg_dtype */
    int32_t rnd;             /* ssg_scale_round of the two moment scales */
    int32_t reserved[3];     /* must be zero */
} ssg_adam_desc;
typedef struct {
    const uint8_t *m_q, *v_q;   /* [n] E4M3 / E5M2 codes */
    const float *scales;        /* [0]=scale_m [1]=scale_v [2]=amax_m [3]=amax_v as written by step `step` */
} ssg_adam_state_view;
size_t ssg_adam_state_bytes(int64_t n);
ssg_status ssg_adam_init(int64_t n, void *state, void *stream);
ssg_status ssg_adam_step(const ssg_adam_desc *desc, const void *grad, float *w, void *w_bf16, void *state,
                         void *stream);
/* pointers into `state` as left by step `step` (0 = after ssg_adam_init) */
ssg_status ssg_adam_view_state(int64_t n, int32_t step, const void *state, ssg_adam_state_view *out);

/* ---- kernel timing for benchmarks (optional) --------------------------------
 * The one piece of state the library keeps, off by default.  While enabled, every kernel launch of the
 * library is bracketed by two HIP events recorded on the launch's own stream (events are host objects; no
 * device memory is allocated).
 *   ssg_profile_enable(n)  n > 0: create n event pairs and start recording (records beyond n are
 *                          dropped); n = 0: stop and destroy the events.
 *   ssg_profile_select(t)  record only launches with tag t (so that the brackets do not perturb the other
 *                          kernels of a timed region); t < 0 = every launch (the default).  Survives
 *                          ssg_profile_enable.
 *   ssg_profile_read       waits for the recorded events, writes up to `cap` durations in milliseconds, their
 *                          tags and (bytes may be NULL) the algorithmic bytes of each launch (host arrays),
 *                          clears the record list and returns the number written, or a negative ssg_status.
 * Tags.  GEMMs (bytes = 0: priced in flops by the caller): 2 * epilogue + a_fmt with epilogue 0 = plain store
 * (y: tag 0; a weight gradient: tag 1), 1 = fused SwiGLU forward (U, G, channel maxima: tag 2), 2 = fused SwiGLU
 * backward (dH: tag 5), 3 = fused SwiGLU product + E4M3 cast of the inference form (tag 6); 11 = the input
 * gradient, both products in one launch (9 and 10: its two launches on shapes where that form is not built);
 * 16 = grouped launch {dH, dW3}; 17 = grouped launch {dX, dW1, dW2}; 18 = tag 2 with the per-column range pass over
 * W3 riding in the same grid; bf16 operands (w3_layer_bf16 = 1): 20 = plain
 * store (y, dW3), 21 = dH with the fused SwiGLU backward.
 * Elementwise passes (bytes = algorithmic bytes moved): 40 = per-tensor range, 41 = per-tensor cast, 42 = cast
 * of the SwiGLU product from bf16 U, G with per-channel factors, 43 = cast of W3 with the inverse factors folded
 * in, 44 = per-column range, 45 = small bookkeeping kernels (resets, factors, history update), 46 = bf16 transposes
 * (w3_layer_bf16 = 1), 47 = the passes of 42 and 43 in one launch.
 * Adam: 32 = range pass, 33 = update pass. */
ssg_status ssg_profile_enable(int max_records);
ssg_status ssg_profile_select(int tag);
int ssg_profile_read(float *ms, int *tags, double *bytes, int cap);

#ifdef __cplusplus
}
#endif
#endif /* SSG_H */
