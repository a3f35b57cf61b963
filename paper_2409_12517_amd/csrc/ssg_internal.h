// Internal launch interface between the C-ABI layer and the kernels.
// Everything takes raw device pointers and a hipStream_t; nothing allocates.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssg {

enum SrcKind { SRC_BF16 = 0, SRC_F32 = 1, SRC_SWIGLU = 2 };

// ---- elementwise / reduction passes (ssg_quant.hip) -------------------------
void launch_fill_u32(uint32_t *p, size_t n, uint32_t value, hipStream_t st);
// zero scalar slots selected by mask (bit i -> scalars[i], i < 32) and two vectors (either may be empty)
void launch_reset(uint32_t *scalars, uint32_t mask, uint32_t *v1, size_t n1, uint32_t *v2, size_t n2, hipStream_t st);

// Running maxima of |x| as float bits, spread over `slots` words that are kAmaxSlotStride words
// (one cache line) apart and must be zeroed by the caller: workgroup b folds into slot b % slots.
// Same-address atomics serialise in L2 (~12 ns each), so a pass that wants thousands of workgroups
// for bandwidth uses kAmaxSlots slots and the consumer takes the maximum over them; slots = 1 is
// the plain single-word form of the public entry points.
constexpr int kAmaxSlots = 64;
constexpr int kAmaxSlotStride = 32;
constexpr size_t kAmaxSlotWords = (size_t)kAmaxSlots * kAmaxSlotStride;
void launch_amax(const void *src, SrcKind kind, size_t n, uint32_t *amax_bits, int slots, hipStream_t st);
// up to three bf16 tensors in one launch, each into its own kAmaxSlots slotted words
void launch_amax_batch(const void *const *src, const size_t *n, uint32_t *const *amax_bits, int count, hipStream_t st);

struct CastArgs {
    const void *src = nullptr;       // bf16 / f32 [rows, cols]; U for SRC_SWIGLU
    const void *src2 = nullptr;      // G for SRC_SWIGLU
    SrcKind kind = SRC_BF16;
    int64_t rows = 0, cols = 0;
    int fmt = 0;                     // kE4M3 / kE5M2
    const float *col_scale = nullptr;   // optional per-column factor applied first (one fp32 multiply)
    const float *amax = nullptr;     // per-tensor: scale = scale_from_amax(max over amax_slots slots) ...
    int amax_slots = 1;
    float *amax_out = nullptr;       // where the reduced amax is recorded (may be null)
    const float *scale_in = nullptr; // ... or a given scale; both null = no per-tensor factor
    int pow2 = 0;
    float *scale_out = nullptr;      // where the per-tensor scale is recorded (may be null)
    uint32_t *record = nullptr;      // optional kAmaxSlots slotted words: max |src| seen by this pass is folded in
                                     // (bf16 source, no per-column factor, transposed copy requested)
    uint8_t *dst = nullptr;          // [rows, cols]
    uint8_t *dst_t = nullptr;        // [cols, rows] or null
    unsigned long long *counters = nullptr;   // optional (no transposed copy): [0] += elements beyond the format's
                                     // range under the scale (saturated), [1] += nonzero elements cast to +-0
};
void launch_cast(const CastArgs &a, hipStream_t st);
// up to three casts of the same form (source kind, format, optional parts) in one launch; others are launched singly
void launch_cast_batch(const CastArgs *list, int n, hipStream_t st);
// the smooth cast of h (from bf16 U, G) and the fold + cast of w3 in one launch (falls back to two for any other pair)
void launch_cast_h_w3(const CastArgs &h, const CastArgs &w3, hipStream_t st);

// camax_bits[c] = max_r |v[r,c]| as float bits (zeroed by the caller).
void launch_col_amax(const void *src, const void *src2, SrcKind kind, int64_t rows, int64_t cols,
                     uint32_t *camax_bits, hipStream_t st);

// Per-channel factors from the per-channel maxima (Section 4.4) and the range
// of s^-1 * w3 for the folded weight.  smooth = 0: one factor for all channels.
//   hmax_bits: scratch for the plain mode (zeroed by the caller); receives the tensor's range
//   h_scale_given: plain mode only, optional device scalar: the scale of h as the caller gives it
void launch_channel_factors(const float *h_camax, const float *w3_camax, int64_t f, int smooth,
                            float *s, float *sinv, uint32_t *amax_w3s_bits, uint32_t *hmax_bits,
                            const float *h_scale_given, hipStream_t st);

// amax_bits = max_i fl32(w3_camax[i] * sinv[i]) as float bits (zeroed by the caller).
void launch_fold_range(const float *w3_camax, const float *sinv, int64_t f, uint32_t *amax_bits, hipStream_t st);

void launch_swiglu(const void *U, const void *G, int64_t n, float *h, hipStream_t st);

// bf16 [rows, cols] -> transposed copy [cols, rows]; and the SwiGLU product of bf16 U, G [rows, cols] rounded once to
// bf16, as it stands (h) and transposed (h_t) -- the operands of the last linear layer when it is left in bf16
void launch_transpose_bf16(const void *src, int64_t rows, int64_t cols, void *dst_t, hipStream_t st);
void launch_swiglu_bf16(const void *U, const void *G, int64_t rows, int64_t cols, void *h, void *h_t, hipStream_t st);

// Q_E4M3 of a bf16 [rows, cols] matrix whose row i is first multiplied by row_scale[i]; `slots` are
// kAmaxSlots zeroed slotted range words (scratch)
void launch_rowscale_quantize(const void *w, const float *row_scale, int64_t rows, int64_t cols, uint32_t *slots,
                              int pow2, float *scale_out, float *amax_out, uint8_t *dst, hipStream_t st);

// ---- FP8 MFMA GEMM (ssg_gemm.hip) --------------------------------------------
enum Epilogue {
    EPI_STORE = 0,        // C = acc * alpha [* col_scale[n]]
    EPI_SWIGLU = 1,       // dual B: U, G bf16 stores + per-channel max of |h|
    EPI_SWIGLU_BWD = 2,   // acc -> dH; loads U, G; stores dU, dG bf16 + their amax
    EPI_SWIGLU_Q = 3,     // dual B as EPI_SWIGLU, but stores only the E4M3 cast of u * Swish(g) (C: bytes [M, N])
    EPI_SWIGLU_BWD_Q = 4  // as EPI_SWIGLU_BWD, but dU, dG leave as E5M2 codes under given scales (C, C2: bytes [M, N]):
                          // code = satcast(fl32(bf16(dU) * q_scale)); the scales are copied to q_scale_out / q_scale_out2
};

struct GemmArgs {
    int epilogue = EPI_STORE;
    int a_fmt = 0;                      // kE4M3 / kE5M2 (B is always E4M3); kBF16 = 2: A and B are bf16 (layout 0,
                                        // EPI_STORE or EPI_SWIGLU_BWD only; K counts elements)
    int64_t M = 0, N = 0, K = 0;
    const uint8_t *A = nullptr;         // [M, K]   (layout 2: stored K-major, [K, M])
    const uint8_t *B = nullptr;         // [N, K]   (layout 1, 2: stored K-major, [K, N])
    int layout = 0;                     // 0 = both K-contiguous; 1 = B K-major; 2 = A and B K-major (EPI_STORE, EPI_SWIGLU_BWD)
    const uint8_t *B2 = nullptr;        // EPI_SWIGLU, EPI_SWIGLU_Q: the second weight matrix [N, K]
    // EPI_STORE as one half of a sum of two products run as two launches:
    //   part = 1: C is the fp32 scratch [M, N] that receives this product, scaled (c_f32 = 1)
    //   part = 2: `add` (that scratch) is added to this product, scaled, before rounding into C
    //   part = 3: the whole sum in one launch: C = A B^T / (sa sb) + A_ph2 B_ph2^T / (sa_ph2 sb_ph2), the second pair of
    //             operands of the same shapes, formats and layout; all four scale pointers are required
    // (parts are built for the input gradient: A E5M2, layout 1)
    int part = 0;
    const float *add = nullptr;
    const uint8_t *A_ph2 = nullptr, *B_ph2 = nullptr;
    const float *sa_ph2 = nullptr, *sb_ph2 = nullptr;
    // dequantization: alpha = 1 / (sa * sb); null pointer = 1
    const float *sa = nullptr, *sb = nullptr, *sb2 = nullptr;   // sb2: scale of B2
    const float *col_scale = nullptr;   // optional [N] factor (EPI_STORE, EPI_SWIGLU_BWD)
    void *C = nullptr;                  // EPI_STORE: [M,N];  EPI_SWIGLU: U;  EPI_SWIGLU_BWD: dU
    void *C2 = nullptr;                 // EPI_SWIGLU: G;  EPI_SWIGLU_BWD: dG
    int c_f32 = 0;                      // EPI_STORE: 1 = fp32 output, 0 = bf16
    const void *U = nullptr, *G = nullptr;      // EPI_SWIGLU_BWD inputs (bf16 [M,N])
    uint32_t *camax_bits = nullptr;     // EPI_SWIGLU: [N] running max |h| (float bits)
    uint32_t *amax_bits = nullptr;      // EPI_SWIGLU_BWD: running max |dU| (float bits), kAmaxSlots slots
    uint32_t *amax_bits2 = nullptr;     //                 same for |dG|
    const float *q_scale = nullptr, *q_scale2 = nullptr;          // EPI_SWIGLU_BWD_Q: scales of dU, dG (device)
    float *q_scale_out = nullptr, *q_scale_out2 = nullptr;        //                   where the scales used are recorded
    void *keep_u = nullptr, *keep_g = nullptr;                    //                   optional bf16 [M,N]: the rounded dU, dG
                                                                  //                   the codes were cast from (both or neither)
    // EPI_SWIGLU, optional: an independent per-column range pass over a bf16 matrix [tail_rows, tail_cols] (columns a
    // multiple of 8) run by extra workgroups at the end of the grid, where they fill the compute units that the last,
    // partly occupied round of tiles leaves idle; tail_camax_bits [tail_cols] (float bits, zeroed by the caller)
    const void *tail_src = nullptr;
    int64_t tail_rows = 0, tail_cols = 0;
    uint32_t *tail_camax_bits = nullptr;
};
// Whether the argument set is one the kernels are built for (part / add / epilogue / layout combinations).
bool gemm_args_ok(const GemmArgs &a);
// false (nothing launched): gemm_args_ok(a) is false
bool launch_gemm(const GemmArgs &a, hipStream_t st);
bool launch_gemm_bwd(const GemmArgs &a, hipStream_t st);       // the backward forms (called by launch_gemm)
bool gemm_sum_in_one_launch_ok(int64_t N, int64_t K);           // shapes for which part = 3 is built
int gemm_profile_tag(const GemmArgs &a);
// Several independent GEMMs in one grid, the workgroups of one following those of the other.  Built groups:
//   { dH (EPI_SWIGLU_BWD or _Q), weight gradient (EPI_STORE, layout 2, A E5M2) }
//   { input gradient as one launch (part = 3), one to three weight gradients }
// gemm_group_ok tells whether `list` is one of them with every member valid; launch_gemm_group returns false
// (nothing launched) otherwise.  Timing tags: 16 and 17.
// split_sets >= 0 splits the LAST member (workgroups come in sets of 8 tiles, gemm_tile_sets of them per GEMM): the
// two-member group runs its sets [0, split_sets), the other group the rest, so that one weight gradient can be
// shared out between the two launches; split_sets < 0: every member whole.
// gemm_group_split_sets picks that split for {dh, dw_split} followed by {second..., rest of dw_split} on `units`
// compute units, from a replay of the in-order dispatch with per-tile times estimated from K steps and epilogues.
bool gemm_group_ok(const GemmArgs *const *list, int n);
bool launch_gemm_group(const GemmArgs *const *list, int n, int split_sets, hipStream_t st);
int gemm_tile_sets(const GemmArgs &a);
int gemm_group_split_sets(const GemmArgs &dh, const GemmArgs &dw_split, const GemmArgs *const *second, int n_second, int units);

// Benchmark hook: called by the launchers before and after a kernel launch (no-ops unless enabled).  `bytes`: the
// algorithmic bytes the launch moves (elementwise passes) or its algorithmic flops (GEMMs).
void profile_before(int tag, hipStream_t st, double bytes = 0.0);
void profile_after(hipStream_t st);
// tags of the elementwise passes (the GEMM tags are listed with ssg_profile_read)
constexpr int kTagAmax = 40, kTagCast = 41, kTagCastSwiglu = 42, kTagCastColscale = 43, kTagColAmax = 44, kTagSmall = 45,
              kTagTranspose = 46, kTagCastHW3 = 47;

// ---- delayed scaling: amax history per tensor (ssg_quant.hip) ----------------------
// State words: tensor k (0..5 = x, w1, w2, dy, du, dg) owns words [32k, 32k+32): [0] the scale the next
// call uses (float), [1] position in the history ring, [2] the range seen in the last call (float),
// [8, 8+kScalingHistory) the ring of ranges.  From word kScalingHeaderWords on: four slotted range
// accumulators (x, w1, w2, dy) of kAmaxSlotWords words each, zero between calls.
constexpr int kScalingTensors = 6, kScalingHistory = 16, kScalingStride = 32;
constexpr size_t kScalingHeaderWords = 256;
constexpr size_t kScalingWords = kScalingHeaderWords + 4 * kAmaxSlotWords;
struct ScalingUpdate {
    uint32_t *slots[3] = {nullptr, nullptr, nullptr};   // slotted range words of the call just made (cleared afterwards)
    int tensor[3] = {0, 0, 0};
    int fmt[3] = {0, 0, 0};
    int count = 0;
    int pow2 = 0;
};
void launch_scaling_init(uint32_t *state, hipStream_t st);
void launch_scaling_update(uint32_t *state, const ScalingUpdate &u, hipStream_t st);

// ---- Adam with FP8 moments (ssg_adam.hip) ---------------------------------------
struct AdamArgs {
    const void *grad = nullptr;      // [n] fp32 or bf16
    int grad_bf16 = 0;
    float *w = nullptr;              // [n] fp32 master weights, updated in place
    void *w_bf16 = nullptr;          // optional [n] bf16 copy of the new weights
    uint8_t *m_q = nullptr, *v_q = nullptr;   // [n] E4M3 / E5M2 codes, updated in place
    uint32_t *scalars = nullptr;     // adam_scalar_words() words
    int64_t n = 0;
    int step = 1;                    // the step being taken (>= 1)
    float beta1 = 0, beta2 = 0, one_minus_beta1 = 0, one_minus_beta2 = 0, c1 = 1, c2 = 1;
    float lr = 0, eps = 0, weight_decay = 0;
    int pow2 = 0;
};
size_t adam_scalar_words();
void launch_adam_init(uint32_t *scalars, uint8_t *codes, size_t code_bytes, hipStream_t st);
void launch_adam_step(const AdamArgs &a, hipStream_t st);

}  // namespace ssg
