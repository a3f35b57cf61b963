// C ABI of libssg.so: argument validation, buffer layouts and the order of the
// passes of the forward and backward block.  Host code only; every step of the
// method runs in the kernels of ssg_quant.hip / ssg_gemm.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/ssg.h"
#include "ssg_device.h"
#include "ssg_internal.h"

namespace {

thread_local char g_err[512] = "";

ssg_status fail(ssg_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Grouped launches of the backward GEMMs are on unless the environment says SSG_GEMM_GROUPING=0 (read once; a
// switch for A/B timing, the results are the same either way).
bool gemm_grouping_enabled() {
    static const bool on = [] { const char *e = std::getenv("SSG_GEMM_GROUPING"); return !(e && e[0] == '0'); }();
    return on;
}

// Shapes, formats and layouts of the five GEMM launches of the backward pass (a10, a12, a13, a14): everything that
// decides how many tiles they have and what a tile costs.  Operand and result pointers are filled in by ssg_mlp_bwd.
struct BackwardGemms { ssg::GemmArgs dh, dw3, dx, dw1, dw2; };
void backward_gemm_shapes(const ssg_mlp_desc &desc, BackwardGemms &b) {
    const int64_t T = desc.T, dm = desc.d, f = desc.f;
    const int dw_f32 = desc.dw_dtype == SSG_F32;
    // a10: dH = s_i * dY^ w3~ / (sdy sw3), then through the SwiGLU product; B = w3~ as stored, [d,f] = [K,N]
    b.dh.epilogue = desc.scale_mode == SSG_SCALE_DELAYED ? ssg::EPI_SWIGLU_BWD_Q : ssg::EPI_SWIGLU_BWD;
    b.dh.a_fmt = ssg::kE5M2; b.dh.M = T; b.dh.N = f; b.dh.K = dm; b.dh.layout = 1;
    // a12: dW3[j,i] = sinv_i * sum_t dY^[t,j] h^[t,i] / sdy; dY^ [T,d] = [K,M], h^ [T,f] = [K,N]
    b.dw3.epilogue = ssg::EPI_STORE; b.dw3.a_fmt = ssg::kE5M2; b.dw3.M = dm; b.dw3.N = f; b.dw3.K = T; b.dw3.layout = 2;
    b.dw3.c_f32 = dw_f32;
    // a13: dX = dU^ w1^ / (sdu sw1) + dG^ w2^ / (sdg sw2); w1^ [f,d] = [K,N]
    b.dx.epilogue = ssg::EPI_STORE; b.dx.a_fmt = ssg::kE5M2; b.dx.M = T; b.dx.N = dm; b.dx.K = f; b.dx.layout = 1;
    b.dx.part = ssg::gemm_sum_in_one_launch_ok(dm, f) ? 3 : 1;
    b.dx.c_f32 = b.dx.part == 3 ? desc.y_dtype == SSG_F32 : 1;
    // a14: dW1 = dU^T x^ / (sdu sx), dW2 = dG^T x^ / (sdg sx); dU^ [T,f] = [K,M], x^ [T,d] = [K,N]
    b.dw1.epilogue = ssg::EPI_STORE; b.dw1.a_fmt = ssg::kE5M2; b.dw1.M = f; b.dw1.N = dm; b.dw1.K = T; b.dw1.layout = 2;
    b.dw1.c_f32 = dw_f32;
    b.dw2 = b.dw1;
    if (desc.w3_layer_bf16) {
        // Section 4.3: dH = dY W3 and dW3 = dY^T h_b on bf16 operands, every operand with its contraction index contiguous
        b.dh.epilogue = ssg::EPI_SWIGLU_BWD; b.dh.a_fmt = ssg::kBF16; b.dh.layout = 0;
        b.dw3.a_fmt = ssg::kBF16; b.dw3.layout = 0;
    }
}

// Split of dW3 between the two grouped launches of the backward (see gemm_group_split_sets), remembered for the last
// few problem shapes: the replay costs a few milliseconds of host time.
int dw3_split_sets(const ssg::GemmArgs &dh, const ssg::GemmArgs &dw3, const ssg::GemmArgs *const *second) {
    struct Entry { int64_t M, N, K; int epilogue, c_f32, device, split; };
    static std::mutex mu;
    static Entry cache[8];
    static int used = 0, next = 0;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return ssg::gemm_tile_sets(dw3);
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i) {
        const Entry &e = cache[i];
        if (e.M == dh.M && e.N == dh.N && e.K == dh.K && e.epilogue == dh.epilogue && e.c_f32 == dw3.c_f32 && e.device == device)
            return e.split;
    }
    int units = 0;
    if (hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) units = 0;
    const int split = ssg::gemm_group_split_sets(dh, dw3, second, 3, units);
    cache[next] = Entry{dh.M, dh.N, dh.K, dh.epilogue, dw3.c_f32, device, split};
    next = (next + 1) % 8;
    used = used < 8 ? used + 1 : 8;
    return split;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool extent_ok(int64_t v) { return v > 0 && (v % 16) == 0; }
constexpr int64_t kMaxElems = (int64_t)1 << 32;   // kernels address operand tiles with 32-bit byte offsets

ssg_status check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SSG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return SSG_OK;
}

// An error some earlier HIP call of the process left behind would otherwise be reported as this entry
// point's own launch failure: it is read (which clears it) and reported before anything is enqueued.
ssg_status check_entry(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(SSG_ERR_HIP, "%s: a HIP error was already pending on entry (%s); nothing was launched", what,
                    hipGetErrorString(e));
    return SSG_OK;
}

#define SSG_REQUIRE_PTR(p)                                                                     \
    do {                                                                                       \
        if ((p) == nullptr) return fail(SSG_ERR_ARG, "%s: %s is NULL", __func__, #p);          \
        if (!aligned16(p)) return fail(SSG_ERR_ARG, "%s: %s is not 16-byte aligned", __func__, #p); \
    } while (0)
#define SSG_OPTIONAL_PTR(p)                                                                    \
    do {                                                                                       \
        if ((p) != nullptr && !aligned16(p))                                                   \
            return fail(SSG_ERR_ARG, "%s: %s is not 16-byte aligned", __func__, #p);           \
    } while (0)
#define SSG_REQUIRE_SCALAR_PTR(p)                                                              \
    do {                                                                                       \
        if ((p) == nullptr) return fail(SSG_ERR_ARG, "%s: %s is NULL", __func__, #p);          \
        if (reinterpret_cast<uintptr_t>(p) & 3u)                                               \
            return fail(SSG_ERR_ARG, "%s: %s is not 4-byte aligned", __func__, #p);            \
    } while (0)

ssg::SrcKind src_kind(ssg_dtype dt) { return dt == SSG_BF16 ? ssg::SRC_BF16 : ssg::SRC_F32; }
bool dtype_ok(int dt) { return dt == SSG_BF16 || dt == SSG_F32; }
bool fmt_ok(int f) { return f == SSG_E4M3 || f == SSG_E5M2; }

// ---- buffer layouts -----------------------------------------------------------
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct SavedLayout {
    size_t scalars, partials, s, sinv, h_camax, w3_camax, x_q, w1_q, w2_q, U, G, h_q, w3_q, h_b, h_bT, w3T, total;
};
// scalar slots of `saved` (floats; amax slots are accumulated as bit patterns)
enum { S_SX = 0, S_SW1, S_SW2, S_SW3, S_AMAX_X, S_AMAX_W1, S_AMAX_W2, S_AMAX_W3S, S_HMAX, S_COUNT = 64 };

SavedLayout saved_layout(const ssg_mlp_desc &d) {
    SavedLayout L;
    const size_t T = d.T, dm = d.d, f = d.f;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
    L.scalars = take(S_COUNT * 4);
    // slotted running maxima of x, W1, W2, then h_camax: zeroed by one contiguous clear
    L.partials = take(3 * ssg::kAmaxSlotWords * 4);
    L.h_camax = take(f * 4); L.w3_camax = take(f * 4);
    L.s = take(f * 4); L.sinv = take(f * 4);
    L.x_q = take(T * dm);
    L.w1_q = take(f * dm); L.w2_q = take(f * dm);
    L.U = take(T * f * 2); L.G = take(T * f * 2);
    L.h_q = take(T * f);
    L.w3_q = take(f * dm);
    // last layer left in bf16 (Section 4.3): the bf16 SwiGLU output, its transposed copy and W3 transposed
    const size_t bf = d.w3_layer_bf16 ? 2 : 0;
    L.h_b = take(T * f * bf); L.h_bT = take(T * f * bf); L.w3T = take(f * dm * bf);
    L.total = o;
    return L;
}

struct WorkLayout { size_t scalars, partials, dy_q, dU, dG, du_q, dg_q, dx_tmp, dyT, total; };
enum { W_SDY = 0, W_SDU, W_SDG, W_AMAX_DY, W_AMAX_DU, W_AMAX_DG, W_COUNT = 64 };

WorkLayout work_layout(const ssg_mlp_desc &d) {
    WorkLayout L;
    const size_t T = d.T, dm = d.d, f = d.f;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
    L.scalars = take(W_COUNT * 4);
    L.partials = take(3 * ssg::kAmaxSlotWords * 4);     // slotted running maxima of dY, dU, dG (adjacent to the scalars)
    L.dy_q = take(T * dm);
    L.dU = take(T * f * 2); L.dG = take(T * f * 2);
    L.du_q = take(T * f); L.dg_q = take(T * f);
    L.dx_tmp = take(T * dm * 4);                        // fp32 first product of the input gradient
    L.dyT = take(d.w3_layer_bf16 ? T * dm * 2 : 0);     // bf16 dY transposed (last layer left in bf16)
    L.total = o;
    return L;
}

ssg_status check_desc(const ssg_mlp_desc *d, const char *who) {
    if (!d) return fail(SSG_ERR_ARG, "%s: desc is NULL", who);
    if (!extent_ok(d->T) || !extent_ok(d->d) || !extent_ok(d->f))
        return fail(SSG_ERR_SHAPE, "%s: T=%lld d=%lld f=%lld must be positive multiples of 16", who,
                    (long long)d->T, (long long)d->d, (long long)d->f);
    if (d->T * d->f >= kMaxElems || d->f * d->d >= kMaxElems || d->T * d->d >= kMaxElems)
        return fail(SSG_ERR_SHAPE, "%s: a matrix of this block has 2^32 or more elements", who);
    if (d->smooth != 0 && d->smooth != 1) return fail(SSG_ERR_ARG, "%s: smooth must be 0 or 1", who);
    if (d->rnd != SSG_ROUND_EXACT_DIV && d->rnd != SSG_ROUND_POW2) return fail(SSG_ERR_ARG, "%s: bad rnd", who);
    if (!dtype_ok(d->y_dtype) || !dtype_ok(d->dw_dtype)) return fail(SSG_ERR_ARG, "%s: bad output dtype", who);
    if (d->weights_cached != 0 && d->weights_cached != 1) return fail(SSG_ERR_ARG, "%s: weights_cached must be 0 or 1", who);
    if (d->scale_mode != SSG_SCALE_CURRENT && d->scale_mode != SSG_SCALE_DELAYED)
        return fail(SSG_ERR_ARG, "%s: scale_mode must be SSG_SCALE_CURRENT or SSG_SCALE_DELAYED", who);
    if (d->scale_mode == SSG_SCALE_DELAYED && d->scaling_state == nullptr)
        return fail(SSG_ERR_ARG, "%s: SSG_SCALE_DELAYED needs scaling_state", who);
    if (d->scaling_state != nullptr && !aligned16(d->scaling_state))
        return fail(SSG_ERR_ARG, "%s: scaling_state is not 16-byte aligned", who);
    if (d->h_scale_mode != SSG_SCALE_CURRENT && d->h_scale_mode != SSG_SCALE_GIVEN)
        return fail(SSG_ERR_ARG, "%s: h_scale_mode must be SSG_SCALE_CURRENT or SSG_SCALE_GIVEN", who);
    if (d->h_scale_mode == SSG_SCALE_GIVEN) {
        if (d->smooth) return fail(SSG_ERR_ARG, "%s: a given scale of h applies to the plain block only (smooth = 0)", who);
        if (d->h_scale == nullptr || (reinterpret_cast<uintptr_t>(d->h_scale) & 3u))
            return fail(SSG_ERR_ARG, "%s: h_scale_mode = SSG_SCALE_GIVEN needs h_scale (device, 4-byte aligned)", who);
    }
    if (d->h_counters != nullptr && (reinterpret_cast<uintptr_t>(d->h_counters) & 7u))
        return fail(SSG_ERR_ARG, "%s: h_counters is not 8-byte aligned", who);
    if (d->keep_bf16_grads != 0 && d->keep_bf16_grads != 1) return fail(SSG_ERR_ARG, "%s: keep_bf16_grads must be 0 or 1", who);
    if (d->w3_layer_bf16 != 0 && d->w3_layer_bf16 != 1) return fail(SSG_ERR_ARG, "%s: w3_layer_bf16 must be 0 or 1", who);
    if (d->w3_layer_bf16) {
        if (d->smooth) return fail(SSG_ERR_ARG, "%s: w3_layer_bf16 = 1 leaves the SwiGLU output unquantized: smooth must be 0", who);
        if (d->scale_mode != SSG_SCALE_CURRENT || d->h_scale_mode != SSG_SCALE_CURRENT)
            return fail(SSG_ERR_UNSUPPORTED, "%s: w3_layer_bf16 = 1 is built for current scaling only", who);
    }
    for (int i = 0; i < 3; ++i)
        if (d->reserved[i] != 0) return fail(SSG_ERR_ARG, "%s: reserved fields must be 0", who);
    return SSG_OK;
}

// ---- optional kernel timing -----------------------------------------------------
struct ProfileState {
    std::vector<hipEvent_t> start, stop;
    std::vector<int> tag;
    std::vector<double> bytes;
    int used = 0;
    int only_tag = -1;       // -1: record every launch; otherwise only launches with this tag
    bool open = false;       // a start event was recorded and waits for its stop
};
ProfileState g_prof;

}  // namespace

namespace ssg {
void profile_before(int tag, hipStream_t st, double bytes) {
    g_prof.open = false;
    if (g_prof.only_tag >= 0 && tag != g_prof.only_tag) return;
    if (g_prof.used >= (int)g_prof.start.size()) return;
    if (hipEventRecord(g_prof.start[g_prof.used], st) != hipSuccess) return;
    g_prof.tag[g_prof.used] = tag;
    g_prof.bytes[g_prof.used] = bytes;
    g_prof.open = true;
}
void profile_after(hipStream_t st) {
    if (!g_prof.open) return;
    g_prof.open = false;
    if (hipEventRecord(g_prof.stop[g_prof.used], st) == hipSuccess) ++g_prof.used;
}
}  // namespace ssg

extern "C" {

ssg_status ssg_profile_select(int tag) {
    g_prof.only_tag = tag < 0 ? -1 : tag;
    return SSG_OK;
}

ssg_status ssg_profile_enable(int max_records) {
    if (max_records < 0 || max_records > (1 << 20)) return fail(SSG_ERR_ARG, "ssg_profile_enable: bad max_records");
    const int keep_tag = g_prof.only_tag;
    for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
    g_prof = ProfileState();
    g_prof.only_tag = keep_tag;
    for (int i = 0; i < max_records; ++i) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess)
            return fail(SSG_ERR_HIP, "ssg_profile_enable: hipEventCreate failed");
        g_prof.start.push_back(a);
        g_prof.stop.push_back(b);
    }
    g_prof.tag.assign((size_t)max_records, 0);
    g_prof.bytes.assign((size_t)max_records, 0.0);
    return SSG_OK;
}

int ssg_profile_read(float *ms, int *tags, double *bytes, int cap) {
    if (!ms || !tags || cap < 0) return fail(SSG_ERR_ARG, "ssg_profile_read: bad argument");
    int n = g_prof.used < cap ? g_prof.used : cap;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms[i], g_prof.start[i], g_prof.stop[i]) != hipSuccess)
            return fail(SSG_ERR_HIP, "ssg_profile_read: event query failed");
        tags[i] = g_prof.tag[i];
        if (bytes) bytes[i] = g_prof.bytes[i];
    }
    g_prof.used = 0;
    return n;
}

// ---- inference with the factors folded into the weights ---------------------------
namespace {
// prepared: scalars (64 floats: [0] s1 [1] s2 [2] s3 [4] amax of s*w1 [5] amax_w2 [6] amax of s^-1*w3),
// three slotted range accumulators, w3's per-channel ranges, then the three code matrices
struct InferPrepared {
    size_t scalars, slots, w3_camax, w1_q, w2_q, w3_q, total;
};
InferPrepared infer_prepared_layout(int64_t d, int64_t f) {
    InferPrepared L;
    size_t off = 0;
    L.scalars = off; off += 256;
    L.slots = off; off += 3 * ssg::kAmaxSlotWords * 4;
    L.w3_camax = off; off = align256(off + (size_t)f * 4);
    L.w1_q = off; off = align256(off + (size_t)f * d);
    L.w2_q = off; off = align256(off + (size_t)f * d);
    L.w3_q = off; off = align256(off + (size_t)f * d);
    L.total = off;
    return L;
}
// workspace: scalars ([0] sx [1] amax_x), one slotted range accumulator, x^ [T,d], h^ [T,f]
struct InferWork {
    size_t scalars, slots, x_q, h_q, total;
};
InferWork infer_work_layout(int64_t T, int64_t d, int64_t f) {
    InferWork L;
    size_t off = 0;
    L.scalars = off; off += 256;
    L.slots = off; off += ssg::kAmaxSlotWords * 4;
    L.x_q = off; off = align256(off + (size_t)T * d);
    L.h_q = off; off = align256(off + (size_t)T * f);
    L.total = off;
    return L;
}
ssg_status check_infer_desc(const ssg_mlp_desc *d, const char *who) {
    ssg_status rc = check_desc(d, who);
    if (rc != SSG_OK) return rc;
    if (d->smooth != 1) return fail(SSG_ERR_UNSUPPORTED, "%s: the folded form is Smooth-SwiGLU (smooth = 1)", who);
    if (d->scale_mode != SSG_SCALE_CURRENT) return fail(SSG_ERR_UNSUPPORTED, "%s: current scaling of x only", who);
    return SSG_OK;
}
}  // namespace

size_t ssg_infer_prepared_bytes(const ssg_mlp_desc *desc) {
    if (check_infer_desc(desc, "ssg_infer_prepared_bytes") != SSG_OK) return 0;
    return infer_prepared_layout(desc->d, desc->f).total;
}
size_t ssg_infer_workspace_bytes(const ssg_mlp_desc *desc) {
    if (check_infer_desc(desc, "ssg_infer_workspace_bytes") != SSG_OK) return 0;
    return infer_work_layout(desc->T, desc->d, desc->f).total;
}

ssg_status ssg_infer_prepare(const ssg_mlp_desc *desc, const void *W1, const void *W2, const void *W3, const float *s,
                             const float *sinv, void *prepared, size_t prepared_bytes, void *stream) {
    ssg_status rc = check_infer_desc(desc, "ssg_infer_prepare");
    if (rc != SSG_OK) return rc;
    SSG_REQUIRE_PTR(W1); SSG_REQUIRE_PTR(W2); SSG_REQUIRE_PTR(W3); SSG_REQUIRE_PTR(s); SSG_REQUIRE_PTR(sinv);
    SSG_REQUIRE_PTR(prepared);
    hipStream_t st = (hipStream_t)stream;
    const int64_t dm = desc->d, f = desc->f;
    const int pow2 = desc->rnd == SSG_ROUND_POW2;
    const InferPrepared L = infer_prepared_layout(dm, f);
    if (prepared_bytes < L.total)
        return fail(SSG_ERR_WORKSPACE, "ssg_infer_prepare: prepared holds %zu bytes, %zu needed", prepared_bytes, L.total);
    if ((rc = check_entry("ssg_infer_prepare")) != SSG_OK) return rc;
    uint8_t *b = static_cast<uint8_t *>(prepared);
    float *sc = reinterpret_cast<float *>(b + L.scalars);
    uint32_t *slots = reinterpret_cast<uint32_t *>(b + L.slots);
    float *w3_camax = reinterpret_cast<float *>(b + L.w3_camax);
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(b), (L.w1_q - L.scalars) / 4, 0u, st);
    // w1~ = Q(s_i * w1_i): the factor goes into row i of w1 (end of Section 4.4)
    ssg::launch_rowscale_quantize(W1, s, f, dm, slots, pow2, sc + 0, sc + 4, b + L.w1_q, st);
    // w2^ = Q(w2)
    ssg::launch_amax(W2, ssg::SRC_BF16, (size_t)(f * dm), slots + ssg::kAmaxSlotWords, ssg::kAmaxSlots, st);
    ssg::CastArgs c;
    c.src = W2; c.kind = ssg::SRC_BF16; c.rows = f; c.cols = dm; c.fmt = ssg::kE4M3; c.pow2 = pow2;
    c.amax = reinterpret_cast<float *>(slots + ssg::kAmaxSlotWords); c.amax_slots = ssg::kAmaxSlots;
    c.amax_out = sc + 5; c.scale_out = sc + 1; c.dst = b + L.w2_q;
    ssg::launch_cast(c, st);
    // w3~ = Q(s_i^-1 * w3_i): column i of the stored [d,f] matrix
    ssg::launch_col_amax(W3, nullptr, ssg::SRC_BF16, dm, f, reinterpret_cast<uint32_t *>(w3_camax), st);
    ssg::launch_fold_range(w3_camax, sinv, f, reinterpret_cast<uint32_t *>(sc + 6), st);
    ssg::CastArgs w;
    w.src = W3; w.kind = ssg::SRC_BF16; w.rows = dm; w.cols = f; w.fmt = ssg::kE4M3; w.pow2 = pow2;
    w.col_scale = sinv; w.amax = sc + 6; w.scale_out = sc + 2; w.dst = b + L.w3_q;
    ssg::launch_cast(w, st);
    return check_launch("ssg_infer_prepare");
}

namespace {
// The forward of the folded form on a workspace that holds infer_work_layout(T, d, f).total bytes; shared by
// ssg_infer_fwd (caller's workspace) and ssg_infer_fwd_noalloc (the library's static device array).
ssg_status infer_forward(const char *who, const ssg_mlp_desc *desc, const void *x, const void *prepared, void *y,
                         uint8_t *wk, hipStream_t st) {
    const int64_t T = desc->T, dm = desc->d, f = desc->f;
    const InferPrepared P = infer_prepared_layout(dm, f);
    const InferWork Wl = infer_work_layout(T, dm, f);
    const uint8_t *pb = static_cast<const uint8_t *>(prepared);
    const float *psc = reinterpret_cast<const float *>(pb + P.scalars);
    float *wsc = reinterpret_cast<float *>(wk + Wl.scalars);
    uint32_t *slots = reinterpret_cast<uint32_t *>(wk + Wl.slots);
    // both inner products, the SwiGLU product and its cast in one kernel: h^ = cast((s_i u_i) Swish(g_i))
    ssg::GemmArgs g;
    g.epilogue = ssg::EPI_SWIGLU_Q; g.a_fmt = ssg::kE4M3; g.M = T; g.N = f; g.K = dm;
    g.A = wk + Wl.x_q; g.B = pb + P.w1_q; g.B2 = pb + P.w2_q; g.sa = wsc + 0; g.sb = psc + 0; g.sb2 = psc + 1;
    g.C = wk + Wl.h_q;
    // y = h^ w3~^T / sigma_w3
    ssg::GemmArgs g2;
    g2.epilogue = ssg::EPI_STORE; g2.a_fmt = ssg::kE4M3; g2.M = T; g2.N = dm; g2.K = f;
    g2.A = wk + Wl.h_q; g2.B = pb + P.w3_q; g2.sb = psc + 2; g2.C = y; g2.c_f32 = desc->y_dtype == SSG_F32;
    if (!ssg::gemm_args_ok(g) || !ssg::gemm_args_ok(g2)) return fail(SSG_ERR_ARG, "%s: internal GEMM arguments", who);
    ssg_status rc = check_entry(who);
    if (rc != SSG_OK) return rc;
    // the range slots start at zero (a fill kernel, not a memset: the call may be under graph capture)
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(wk), (Wl.x_q - Wl.scalars) / 4, 0u, st);
    // x^ = Q(x)
    ssg::launch_amax(x, ssg::SRC_BF16, (size_t)(T * dm), slots, ssg::kAmaxSlots, st);
    ssg::CastArgs c;
    c.src = x; c.kind = ssg::SRC_BF16; c.rows = T; c.cols = dm; c.fmt = ssg::kE4M3; c.pow2 = desc->rnd == SSG_ROUND_POW2;
    c.amax = reinterpret_cast<float *>(slots); c.amax_slots = ssg::kAmaxSlots; c.amax_out = wsc + 1; c.scale_out = wsc + 0;
    c.dst = wk + Wl.x_q;
    ssg::launch_cast(c, st);
    ssg::launch_gemm(g, st);
    ssg::launch_gemm(g2, st);
    return check_launch(who);
}

// ---- the workspace of ssg_infer_fwd_noalloc: a static device array, one copy per GPU -------------------
constexpr size_t kNoAllocScratchBytes = (size_t)16 << 20;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
unsigned char *g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each GPU, looked up once
std::mutex g_scratch_mutex;

// The address of this GPU's copy of `scratch` (the array's name is a host-side stand-in, never a device address).
ssg_status scratch_address(const char *who, unsigned char **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(SSG_ERR_HIP, "%s: hipGetDevice failed or device index beyond %d", who, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr)
            return fail(SSG_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", who, hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return SSG_OK;
}
}  // namespace

ssg_status ssg_infer_fwd(const ssg_mlp_desc *desc, const void *x, const void *prepared, size_t prepared_bytes, void *y,
                         void *workspace, size_t workspace_bytes, void *stream) {
    ssg_status rc = check_infer_desc(desc, "ssg_infer_fwd");
    if (rc != SSG_OK) return rc;
    SSG_REQUIRE_PTR(x); SSG_REQUIRE_PTR(prepared); SSG_REQUIRE_PTR(y); SSG_REQUIRE_PTR(workspace);
    const size_t need_p = infer_prepared_layout(desc->d, desc->f).total;
    const size_t need_w = infer_work_layout(desc->T, desc->d, desc->f).total;
    if (prepared_bytes < need_p)
        return fail(SSG_ERR_WORKSPACE, "ssg_infer_fwd: prepared holds %zu bytes, %zu needed", prepared_bytes, need_p);
    if (workspace_bytes < need_w)
        return fail(SSG_ERR_WORKSPACE, "ssg_infer_fwd: workspace holds %zu bytes, %zu needed", workspace_bytes, need_w);
    return infer_forward("ssg_infer_fwd", desc, x, prepared, y, static_cast<uint8_t *>(workspace), (hipStream_t)stream);
}

size_t ssg_infer_noalloc_max_bytes(void) { return kNoAllocScratchBytes; }

ssg_status ssg_infer_fwd_noalloc(const ssg_mlp_desc *desc, const void *x, const void *prepared, size_t prepared_bytes,
                                 void *y, void *stream) {
    ssg_status rc = check_infer_desc(desc, "ssg_infer_fwd_noalloc");
    if (rc != SSG_OK) return rc;
    SSG_REQUIRE_PTR(x); SSG_REQUIRE_PTR(prepared); SSG_REQUIRE_PTR(y);
    const size_t need_p = infer_prepared_layout(desc->d, desc->f).total;
    const size_t need_w = infer_work_layout(desc->T, desc->d, desc->f).total;
    if (prepared_bytes < need_p)
        return fail(SSG_ERR_WORKSPACE, "ssg_infer_fwd_noalloc: prepared holds %zu bytes, %zu needed", prepared_bytes, need_p);
    if (need_w > kNoAllocScratchBytes)
        return fail(SSG_ERR_WORKSPACE,
                    "ssg_infer_fwd_noalloc: T=%lld d=%lld f=%lld needs %zu bytes of scratch, the static array holds %zu "
                    "(use ssg_infer_fwd with a caller-allocated workspace)",
                    (long long)desc->T, (long long)desc->d, (long long)desc->f, need_w, kNoAllocScratchBytes);
    unsigned char *ptr = nullptr;
    if ((rc = scratch_address("ssg_infer_fwd_noalloc", &ptr)) != SSG_OK) return rc;
    return infer_forward("ssg_infer_fwd_noalloc", desc, x, prepared, y, ptr, (hipStream_t)stream);
}

ssg_status ssg_infer_view(const ssg_mlp_desc *desc, const void *prepared, const void *workspace, ssg_infer_view_t *out) {
    ssg_status rc = check_infer_desc(desc, "ssg_infer_view");
    if (rc != SSG_OK) return rc;
    if (!out) return fail(SSG_ERR_ARG, "ssg_infer_view: out is NULL");
    const InferPrepared P = infer_prepared_layout(desc->d, desc->f);
    const InferWork Wl = infer_work_layout(desc->T, desc->d, desc->f);
    const uint8_t *pb = static_cast<const uint8_t *>(prepared), *wb = static_cast<const uint8_t *>(workspace);
    out->weight_scales = pb ? reinterpret_cast<const float *>(pb + P.scalars) : nullptr;
    out->w1_q = pb ? pb + P.w1_q : nullptr; out->w2_q = pb ? pb + P.w2_q : nullptr; out->w3_q = pb ? pb + P.w3_q : nullptr;
    out->x_scale = wb ? reinterpret_cast<const float *>(wb + Wl.scalars) : nullptr;
    out->x_q = wb ? wb + Wl.x_q : nullptr; out->h_q = wb ? wb + Wl.h_q : nullptr;
    return SSG_OK;
}

// ---- Adam with FP8 moments -----------------------------------------------------
namespace {
size_t adam_scalar_bytes() { return align256(ssg::adam_scalar_words() * sizeof(uint32_t)); }
bool adam_n_ok(int64_t n) { return n > 0 && (n % 16) == 0 && n < ((int64_t)1 << 40); }
}  // namespace

size_t ssg_adam_state_bytes(int64_t n) {
    if (!adam_n_ok(n)) return 0;
    return adam_scalar_bytes() + 2 * align256((size_t)n);
}

ssg_status ssg_adam_init(int64_t n, void *state, void *stream) {
    if (!adam_n_ok(n)) return fail(SSG_ERR_SHAPE, "ssg_adam_init: n = %lld must be a positive multiple of 16", (long long)n);
    SSG_REQUIRE_PTR(state);
    uint8_t *base = static_cast<uint8_t *>(state);
    ssg::launch_adam_init(reinterpret_cast<uint32_t *>(base), base + adam_scalar_bytes(), 2 * align256((size_t)n),
                          static_cast<hipStream_t>(stream));
    return check_launch("ssg_adam_init");
}

ssg_status ssg_adam_step(const ssg_adam_desc *desc, const void *grad, float *w, void *w_bf16, void *state,
                         void *stream) {
    if (!desc) return fail(SSG_ERR_ARG, "ssg_adam_step: desc is NULL");
    if (!adam_n_ok(desc->n)) return fail(SSG_ERR_SHAPE, "ssg_adam_step: n = %lld must be a positive multiple of 16", (long long)desc->n);
    if (desc->step < 1) return fail(SSG_ERR_ARG, "ssg_adam_step: step %d (steps count from 1)", desc->step);
    if (!dtype_ok(desc->grad_dtype)) return fail(SSG_ERR_ARG, "ssg_adam_step: grad_dtype %d", desc->grad_dtype);
    if (desc->rnd != SSG_ROUND_EXACT_DIV && desc->rnd != SSG_ROUND_POW2) return fail(SSG_ERR_ARG, "ssg_adam_step: rnd %d", desc->rnd);
    if (desc->reserved[0] || desc->reserved[1] || desc->reserved[2]) return fail(SSG_ERR_ARG, "ssg_adam_step: reserved fields must be zero");
    if (!(desc->beta1 >= 0.0f && desc->beta1 < 1.0f) || !(desc->beta2 >= 0.0f && desc->beta2 < 1.0f))
        return fail(SSG_ERR_ARG, "ssg_adam_step: beta1, beta2 must lie in [0, 1)");
    if (!(desc->eps >= 0.0f) || !(desc->lr == desc->lr) || !(desc->weight_decay == desc->weight_decay))
        return fail(SSG_ERR_ARG, "ssg_adam_step: eps must be >= 0 and lr, weight_decay must be numbers");
    SSG_REQUIRE_PTR(grad);
    SSG_REQUIRE_PTR(w);
    SSG_OPTIONAL_PTR(w_bf16);
    SSG_REQUIRE_PTR(state);
    uint8_t *base = static_cast<uint8_t *>(state);
    ssg::AdamArgs a;
    a.grad = grad; a.grad_bf16 = desc->grad_dtype == SSG_BF16; a.w = w; a.w_bf16 = w_bf16;
    a.scalars = reinterpret_cast<uint32_t *>(base);
    a.m_q = base + adam_scalar_bytes();
    a.v_q = a.m_q + align256((size_t)desc->n);
    a.n = desc->n; a.step = desc->step;
    a.beta1 = desc->beta1; a.beta2 = desc->beta2;
    a.one_minus_beta1 = 1.0f - desc->beta1; a.one_minus_beta2 = 1.0f - desc->beta2;
    // bias corrections: formed in double from the binary32 betas, rounded once
    a.c1 = (float)(1.0 / (1.0 - std::pow((double)desc->beta1, (double)desc->step)));
    a.c2 = (float)(1.0 / (1.0 - std::pow((double)desc->beta2, (double)desc->step)));
    a.lr = desc->lr; a.eps = desc->eps; a.weight_decay = desc->weight_decay; a.pow2 = desc->rnd == SSG_ROUND_POW2;
    ssg::launch_adam_step(a, static_cast<hipStream_t>(stream));
    return check_launch("ssg_adam_step");
}

ssg_status ssg_adam_view_state(int64_t n, int32_t step, const void *state, ssg_adam_state_view *out) {
    if (!adam_n_ok(n) || step < 0 || !state || !out) return fail(SSG_ERR_ARG, "ssg_adam_view_state: bad argument");
    const uint8_t *base = static_cast<const uint8_t *>(state);
    out->scales = reinterpret_cast<const float *>(base) + 8 * (step & 1);
    out->m_q = base + adam_scalar_bytes();
    out->v_q = out->m_q + align256((size_t)n);
    return SSG_OK;
}

const char *ssg_last_error(void) { return g_err; }
const char *ssg_version(void) { return "ssg 0.1 (gfx950)"; }

ssg_status ssg_amax(const void *src, ssg_dtype src_dtype, size_t n, float *amax_dev, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!dtype_ok(src_dtype)) return fail(SSG_ERR_ARG, "ssg_amax: bad src_dtype");
    SSG_REQUIRE_SCALAR_PTR(amax_dev);
    if (n % 16) return fail(SSG_ERR_SHAPE, "ssg_amax: n=%zu must be a multiple of 16", n);
    if (n) SSG_REQUIRE_PTR(src);
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_dev), 1, 0u, st);
    ssg::launch_amax(src, src_kind(src_dtype), n, reinterpret_cast<uint32_t *>(amax_dev), 1, st);
    return check_launch("ssg_amax");
}

ssg_status ssg_quantize(const void *src, ssg_dtype src_dtype, int64_t rows, int64_t cols, ssg_fp8_format fmt,
                        ssg_scale_mode mode, ssg_scale_round rnd, uint8_t *dst, uint8_t *dst_t,
                        float *scale_dev, float *amax_dev, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!dtype_ok(src_dtype)) return fail(SSG_ERR_ARG, "ssg_quantize: bad src_dtype");
    if (!fmt_ok(fmt)) return fail(SSG_ERR_ARG, "ssg_quantize: bad fmt");
    if (mode != SSG_SCALE_CURRENT && mode != SSG_SCALE_GIVEN) return fail(SSG_ERR_ARG, "ssg_quantize: bad mode");
    if (rnd != SSG_ROUND_EXACT_DIV && rnd != SSG_ROUND_POW2) return fail(SSG_ERR_ARG, "ssg_quantize: bad rnd");
    if (rows < 0 || cols < 0 || rows % 16 || cols % 16)
        return fail(SSG_ERR_SHAPE, "ssg_quantize: rows=%lld cols=%lld must be non-negative multiples of 16",
                    (long long)rows, (long long)cols);
    if (rows * cols >= kMaxElems) return fail(SSG_ERR_SHAPE, "ssg_quantize: 2^32 or more elements");
    SSG_REQUIRE_SCALAR_PTR(scale_dev);
    if (mode == SSG_SCALE_CURRENT) SSG_REQUIRE_SCALAR_PTR(amax_dev);
    const bool empty = rows == 0 || cols == 0;
    if (!empty) {
        SSG_REQUIRE_PTR(src);
        SSG_REQUIRE_PTR(dst);
        SSG_OPTIONAL_PTR(dst_t);
    }
    ssg::CastArgs a;
    a.src = src; a.kind = src_kind(src_dtype); a.rows = rows; a.cols = cols; a.fmt = fmt;
    a.dst = dst; a.dst_t = dst_t; a.pow2 = rnd == SSG_ROUND_POW2;
    if (mode == SSG_SCALE_CURRENT) {
        ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_dev), 1, 0u, st);
        ssg::launch_amax(src, a.kind, (size_t)(rows * cols), reinterpret_cast<uint32_t *>(amax_dev), 1, st);
        a.amax = amax_dev;
        a.scale_out = scale_dev;
        if (empty) ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(scale_dev), 1, 0x3f800000u, st);
    } else {
        a.scale_in = scale_dev;
        if (amax_dev && !empty) {
            ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_dev), 1, 0u, st);
            ssg::launch_amax(src, a.kind, (size_t)(rows * cols), reinterpret_cast<uint32_t *>(amax_dev), 1, st);
        }
    }
    ssg::launch_cast(a, st);
    return check_launch("ssg_quantize");
}

ssg_status ssg_gemm_fp8_layout(const uint8_t *A, ssg_fp8_format a_fmt, int a_kmajor, const uint8_t *B,
                               ssg_fp8_format b_fmt, int b_kmajor, int64_t M, int64_t N, int64_t K, const float *sa_dev,
                               const float *sb_dev, void *C, ssg_dtype c_dtype, void *stream) {
    if (!fmt_ok(a_fmt) || !fmt_ok(b_fmt)) return fail(SSG_ERR_ARG, "ssg_gemm_fp8: bad format");
    if (b_fmt != SSG_E4M3) return fail(SSG_ERR_UNSUPPORTED, "ssg_gemm_fp8: B must be E4M3");
    if (!dtype_ok(c_dtype)) return fail(SSG_ERR_ARG, "ssg_gemm_fp8: bad c_dtype");
    if ((a_kmajor != 0 && a_kmajor != 1) || (b_kmajor != 0 && b_kmajor != 1)) return fail(SSG_ERR_ARG, "ssg_gemm_fp8: bad layout flag");
    if (a_kmajor && !b_kmajor) return fail(SSG_ERR_UNSUPPORTED, "ssg_gemm_fp8: A K-major with B K-contiguous is not built");
    if (!extent_ok(M) || !extent_ok(N) || !extent_ok(K))
        return fail(SSG_ERR_SHAPE, "ssg_gemm_fp8: M=%lld N=%lld K=%lld must be positive multiples of 16",
                    (long long)M, (long long)N, (long long)K);
    if (M * K >= kMaxElems || N * K >= kMaxElems || M * N >= kMaxElems)
        return fail(SSG_ERR_SHAPE, "ssg_gemm_fp8: a matrix has 2^32 or more elements");
    SSG_REQUIRE_PTR(A); SSG_REQUIRE_PTR(B); SSG_REQUIRE_PTR(C);
    ssg::GemmArgs g;
    g.epilogue = ssg::EPI_STORE; g.a_fmt = a_fmt; g.M = M; g.N = N; g.K = K; g.A = A; g.B = B;
    g.layout = a_kmajor ? 2 : (b_kmajor ? 1 : 0);
    g.sa = sa_dev; g.sb = sb_dev; g.C = C; g.c_f32 = c_dtype == SSG_F32;
    if (!ssg::gemm_args_ok(g)) return fail(SSG_ERR_ARG, "ssg_gemm_fp8: internal GEMM arguments");
    ssg_status rc = check_entry("ssg_gemm_fp8");
    if (rc != SSG_OK) return rc;
    ssg::launch_gemm(g, (hipStream_t)stream);
    return check_launch("ssg_gemm_fp8");
}

ssg_status ssg_gemm_fp8(const uint8_t *A, ssg_fp8_format a_fmt, const uint8_t *B, ssg_fp8_format b_fmt, int64_t M,
                        int64_t N, int64_t K, const float *sa_dev, const float *sb_dev, void *C,
                        ssg_dtype c_dtype, void *stream) {
    return ssg_gemm_fp8_layout(A, a_fmt, 0, B, b_fmt, 0, M, N, K, sa_dev, sb_dev, C, c_dtype, stream);
}

ssg_status ssg_swiglu(const void *U, const void *G, int64_t T, int64_t f, float *h, void *stream) {
    if (!extent_ok(T) || !extent_ok(f)) return fail(SSG_ERR_SHAPE, "ssg_swiglu: T, f must be positive multiples of 16");
    if (T * f >= kMaxElems) return fail(SSG_ERR_SHAPE, "ssg_swiglu: 2^32 or more elements");
    SSG_REQUIRE_PTR(U); SSG_REQUIRE_PTR(G); SSG_REQUIRE_PTR(h);
    ssg::launch_swiglu(U, G, T * f, h, (hipStream_t)stream);
    return check_launch("ssg_swiglu");
}

ssg_status ssg_smooth_swiglu_quantize(const void *U, const void *G, int64_t T, int64_t f, int smooth, uint8_t *h_q,
                                      uint8_t *h_qT, float *s, float *sinv, float *camax, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!extent_ok(T) || !extent_ok(f))
        return fail(SSG_ERR_SHAPE, "ssg_smooth_swiglu_quantize: T, f must be positive multiples of 16");
    if (T * f >= kMaxElems) return fail(SSG_ERR_SHAPE, "ssg_smooth_swiglu_quantize: 2^32 or more elements");
    if (smooth != 0 && smooth != 1) return fail(SSG_ERR_ARG, "ssg_smooth_swiglu_quantize: smooth must be 0 or 1");
    SSG_REQUIRE_PTR(U); SSG_REQUIRE_PTR(G); SSG_REQUIRE_PTR(h_q); SSG_OPTIONAL_PTR(h_qT);
    SSG_REQUIRE_PTR(s); SSG_REQUIRE_PTR(sinv); SSG_REQUIRE_PTR(camax);
    // The first 16 bytes of h_q serve as scratch until the cast overwrites them: word 0 = running
    // tensor maximum for the plain mode, word 1 = sink for the folded-weight range (unused here).
    uint32_t *hmax = reinterpret_cast<uint32_t *>(h_q);
    uint32_t *sink = hmax + 1;
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(camax), (size_t)f, 0u, st);
    ssg::launch_fill_u32(hmax, 4, 0u, st);
    ssg::launch_col_amax(U, G, ssg::SRC_SWIGLU, T, f, reinterpret_cast<uint32_t *>(camax), st);
    // camax also stands in for the per-channel range of w3 (its product only feeds the sink)
    ssg::launch_channel_factors(camax, camax, f, smooth, s, sinv, sink, hmax, nullptr, st);
    ssg::CastArgs a;
    a.src = U; a.src2 = G; a.kind = ssg::SRC_SWIGLU; a.rows = T; a.cols = f; a.fmt = ssg::kE4M3;
    a.col_scale = s; a.dst = h_q; a.dst_t = h_qT;
    ssg::launch_cast(a, st);
    return check_launch("ssg_smooth_swiglu_quantize");
}

ssg_status ssg_fold_w3(const void *W3, const float *sinv, int64_t d, int64_t f, uint8_t *w3_q, uint8_t *w3_qT,
                       float *w3_camax, float *scale_dev, float *amax_dev, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!extent_ok(d) || !extent_ok(f)) return fail(SSG_ERR_SHAPE, "ssg_fold_w3: d, f must be positive multiples of 16");
    if (d * f >= kMaxElems) return fail(SSG_ERR_SHAPE, "ssg_fold_w3: 2^32 or more elements");
    SSG_REQUIRE_PTR(W3); SSG_REQUIRE_PTR(sinv); SSG_REQUIRE_PTR(w3_q); SSG_OPTIONAL_PTR(w3_qT);
    SSG_REQUIRE_PTR(w3_camax); SSG_REQUIRE_SCALAR_PTR(scale_dev); SSG_REQUIRE_SCALAR_PTR(amax_dev);
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(w3_camax), (size_t)f, 0u, st);
    ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(amax_dev), 1, 0u, st);
    ssg::launch_col_amax(W3, nullptr, ssg::SRC_BF16, d, f, reinterpret_cast<uint32_t *>(w3_camax), st);
    ssg::launch_fold_range(w3_camax, sinv, f, reinterpret_cast<uint32_t *>(amax_dev), st);
    ssg::CastArgs a;
    a.src = W3; a.kind = ssg::SRC_BF16; a.rows = d; a.cols = f; a.fmt = ssg::kE4M3;
    a.col_scale = sinv; a.amax = amax_dev; a.scale_out = scale_dev; a.dst = w3_q; a.dst_t = w3_qT;
    ssg::launch_cast(a, st);
    return check_launch("ssg_fold_w3");
}

size_t ssg_mlp_saved_bytes(const ssg_mlp_desc *desc) {
    if (check_desc(desc, "ssg_mlp_saved_bytes") != SSG_OK) return 0;
    return saved_layout(*desc).total;
}
size_t ssg_mlp_workspace_bytes(const ssg_mlp_desc *desc) {
    if (check_desc(desc, "ssg_mlp_workspace_bytes") != SSG_OK) return 0;
    return work_layout(*desc).total;
}

size_t ssg_mlp_scaling_state_bytes(void) { return align256(ssg::kScalingWords * sizeof(uint32_t)); }

ssg_status ssg_mlp_scaling_init(void *scaling_state, void *stream) {
    SSG_REQUIRE_PTR(scaling_state);
    ssg::launch_scaling_init(static_cast<uint32_t *>(scaling_state), static_cast<hipStream_t>(stream));
    return check_launch("ssg_mlp_scaling_init");
}

ssg_status ssg_mlp_view_saved(const ssg_mlp_desc *desc, const void *saved, ssg_mlp_saved_view *out) {
    ssg_status rc = check_desc(desc, "ssg_mlp_view_saved");
    if (rc != SSG_OK) return rc;
    if (!saved || !out) return fail(SSG_ERR_ARG, "ssg_mlp_view_saved: NULL argument");
    const SavedLayout L = saved_layout(*desc);
    const uint8_t *b = static_cast<const uint8_t *>(saved);
    out->scales = reinterpret_cast<const float *>(b + L.scalars);
    out->s = reinterpret_cast<const float *>(b + L.s);
    out->sinv = reinterpret_cast<const float *>(b + L.sinv);
    out->h_camax = reinterpret_cast<const float *>(b + L.h_camax);
    out->w3_camax = reinterpret_cast<const float *>(b + L.w3_camax);
    out->x_q = b + L.x_q;
    out->w1_q = b + L.w1_q; out->w2_q = b + L.w2_q;
    out->h_q = b + L.h_q; out->w3_q = b + L.w3_q;
    out->U = b + L.U; out->G = b + L.G;
    out->h_b = desc->w3_layer_bf16 ? b + L.h_b : nullptr;
    out->h_bT = desc->w3_layer_bf16 ? b + L.h_bT : nullptr;
    out->w3T = desc->w3_layer_bf16 ? b + L.w3T : nullptr;
    return SSG_OK;
}

ssg_status ssg_mlp_view_workspace(const ssg_mlp_desc *desc, const void *workspace, ssg_mlp_workspace_view *out) {
    ssg_status rc = check_desc(desc, "ssg_mlp_view_workspace");
    if (rc != SSG_OK) return rc;
    if (!workspace || !out) return fail(SSG_ERR_ARG, "ssg_mlp_view_workspace: NULL argument");
    const WorkLayout L = work_layout(*desc);
    const uint8_t *b = static_cast<const uint8_t *>(workspace);
    out->scales = reinterpret_cast<const float *>(b + L.scalars);
    out->dy_q = b + L.dy_q;
    out->du_q = b + L.du_q; out->dg_q = b + L.dg_q;
    out->dU = b + L.dU; out->dG = b + L.dG;
    out->dyT = desc->w3_layer_bf16 ? b + L.dyT : nullptr;
    return SSG_OK;
}

ssg_status ssg_mlp_fwd(const ssg_mlp_desc *desc, const void *x, const void *W1, const void *W2, const void *W3,
                       void *y, void *saved, size_t saved_bytes, void *stream) {
    ssg_status rc = check_desc(desc, "ssg_mlp_fwd");
    if (rc != SSG_OK) return rc;
    SSG_REQUIRE_PTR(x); SSG_REQUIRE_PTR(W1); SSG_REQUIRE_PTR(W2); SSG_REQUIRE_PTR(W3);
    SSG_REQUIRE_PTR(y); SSG_REQUIRE_PTR(saved);
    hipStream_t st = (hipStream_t)stream;
    const int64_t T = desc->T, dm = desc->d, f = desc->f;
    const int pow2 = desc->rnd == SSG_ROUND_POW2;
    const SavedLayout L = saved_layout(*desc);
    if (saved_bytes < L.total)
        return fail(SSG_ERR_WORKSPACE, "ssg_mlp_fwd: saved holds %zu bytes, %zu needed (ssg_mlp_saved_bytes)", saved_bytes, L.total);
    uint8_t *b = static_cast<uint8_t *>(saved);
    float *sc = reinterpret_cast<float *>(b + L.scalars);
    uint32_t *scb = reinterpret_cast<uint32_t *>(sc);
    float *h_camax = reinterpret_cast<float *>(b + L.h_camax), *w3_camax = reinterpret_cast<float *>(b + L.w3_camax);
    float *s = reinterpret_cast<float *>(b + L.s), *sinv = reinterpret_cast<float *>(b + L.sinv);

    // every GEMM argument set is built and checked before the first launch
    // a3 + a4 + first half of a5: both inner products of Eq. 2, bf16 U and G, per-channel max |h|
    ssg::GemmArgs g;
    g.epilogue = ssg::EPI_SWIGLU; g.a_fmt = ssg::kE4M3; g.M = T; g.N = f; g.K = dm;
    g.A = b + L.x_q; g.B = b + L.w1_q; g.B2 = b + L.w2_q;
    g.sa = sc + S_SX; g.sb = sc + S_SW1; g.sb2 = sc + S_SW2;
    g.C = b + L.U; g.C2 = b + L.G; g.camax_bits = reinterpret_cast<uint32_t *>(h_camax);
    // a8: last linear layer.  Smooth: only the scale of w3~ is left; plain: s_i = sigma_h for all i
    ssg::GemmArgs g2;
    g2.epilogue = ssg::EPI_STORE; g2.a_fmt = ssg::kE4M3; g2.M = T; g2.N = dm; g2.K = f;
    g2.A = b + L.h_q; g2.B = b + L.w3_q;
    g2.sa = desc->smooth ? nullptr : s; g2.sb = sc + S_SW3;
    g2.C = y; g2.c_f32 = desc->y_dtype == SSG_F32;
    const bool bf16_last = desc->w3_layer_bf16 != 0;
    if (bf16_last) {
        // Section 4.3: the last linear layer on bf16 operands: y = h_b W3^T, no scales
        g2.a_fmt = ssg::kBF16; g2.A = b + L.h_b; g2.B = static_cast<const uint8_t *>(W3); g2.sa = nullptr; g2.sb = nullptr;
    }
    const bool cached = desc->weights_cached != 0;
    // the per-channel range of w3 (needed for the range of s^-1 * w3, constant between weight updates) rides in the
    // gate/up GEMM's grid, where it fills the last, partly occupied round of tiles
    const bool w3_range_in_gemm = !cached && !bf16_last && gemm_grouping_enabled();
    if (w3_range_in_gemm) {
        g.tail_src = W3; g.tail_rows = dm; g.tail_cols = f; g.tail_camax_bits = reinterpret_cast<uint32_t *>(w3_camax);
    }
    if (!ssg::gemm_args_ok(g) || !ssg::gemm_args_ok(g2)) return fail(SSG_ERR_ARG, "ssg_mlp_fwd: internal GEMM arguments");
    if ((rc = check_entry("ssg_mlp_fwd")) != SSG_OK) return rc;

    // zero the running maxima of this call; with cached weights the slots that belong to W1, W2 and
    // W3 (their scales, ranges and W3's per-channel maxima) are left as the earlier call wrote them
    const uint32_t per_call = (1u << S_AMAX_W3S) | (1u << S_HMAX);
    uint32_t *part = reinterpret_cast<uint32_t *>(b + L.partials);
    uint32_t *part_x = part, *part_w1 = part + ssg::kAmaxSlotWords, *part_w2 = part + 2 * ssg::kAmaxSlotWords;
    ssg::launch_reset(scb, per_call, part, (size_t)((L.h_camax - L.partials) / 4) + (size_t)f,
                      reinterpret_cast<uint32_t *>(w3_camax), cached ? 0 : (size_t)f, st);
    if (desc->h_counters) ssg::launch_fill_u32(reinterpret_cast<uint32_t *>(desc->h_counters), 4, 0u, st);

    // a1 + a2: per-tensor range (Section 2), then Q (Eq. 2); row-major only: the backward contractions
    // read these tensors K-major.  Range and cast of one tensor run back to back so that the second read of
    // the tensor can still be served from the memory-side cache.
    // Delayed scaling (Section 2): the scale comes from the history in the caller's state and the
    // cast itself records the range it sees, so the stand-alone range pass disappears.
    const bool delayed = desc->scale_mode == SSG_SCALE_DELAYED;
    uint32_t *state = static_cast<uint32_t *>(desc->scaling_state);
    auto state_scale = [&](int k) { return reinterpret_cast<float *>(state + (size_t)k * ssg::kScalingStride); };
    auto state_slots = [&](int j) { return state + ssg::kScalingHeaderWords + (size_t)j * ssg::kAmaxSlotWords; };
    // x and (unless cached) W1, W2 go through one range launch and one cast launch together
    ssg::CastArgs casts[3];
    const void *srcs[3]; size_t counts[3]; uint32_t *slot_ptrs[3];
    int n_in = 0;
    auto add_input = [&](const void *src, int64_t rows, int64_t cols, uint32_t *part, int k, float *amax_out,
                         float *scale_out, uint8_t *dst) {
        ssg::CastArgs &c = casts[n_in];
        c.kind = ssg::SRC_BF16; c.fmt = ssg::kE4M3; c.pow2 = pow2; c.amax_slots = ssg::kAmaxSlots;
        c.src = src; c.rows = rows; c.cols = cols; c.scale_out = scale_out; c.dst = dst;
        if (delayed) {
            c.scale_in = state_scale(k); c.record = state_slots(k);
        } else {
            c.amax = reinterpret_cast<float *>(part); c.amax_out = amax_out;
        }
        srcs[n_in] = src; counts[n_in] = (size_t)(rows * cols); slot_ptrs[n_in] = part;
        ++n_in;
    };
    add_input(x, T, dm, part_x, 0, sc + S_AMAX_X, sc + S_SX, b + L.x_q);
    if (!cached) {
        add_input(W1, f, dm, part_w1, 1, sc + S_AMAX_W1, sc + S_SW1, b + L.w1_q);
        add_input(W2, f, dm, part_w2, 2, sc + S_AMAX_W2, sc + S_SW2, b + L.w2_q);
    }
    if (!delayed) ssg::launch_amax_batch(srcs, counts, slot_ptrs, n_in, st);
    ssg::launch_cast_batch(casts, n_in, st);
    if (!cached) {
        // per-channel range of w3 as a launch of its own (unless it rides in the GEMM below)
        if (!bf16_last && !w3_range_in_gemm)
            ssg::launch_col_amax(W3, nullptr, ssg::SRC_BF16, dm, f, reinterpret_cast<uint32_t *>(w3_camax), st);
        // last layer in bf16: its input gradient contracts over d, so W3 [d,f] is also kept transposed
        if (bf16_last) ssg::launch_transpose_bf16(W3, dm, f, b + L.w3T, st);
    }

    ssg::launch_gemm(g, st);

    if (bf16_last) {
        // the SwiGLU output stays in bf16 (rounded once from the fp32 product), straight and transposed
        ssg::launch_swiglu_bf16(b + L.U, b + L.G, T, f, b + L.h_b, b + L.h_bT, st);
        ssg::launch_gemm(g2, st);
        if (state) {
            ssg::ScalingUpdate u;
            u.pow2 = pow2;
            u.slots[0] = part_x; u.tensor[0] = 0; u.fmt[0] = ssg::kE4M3; u.count = 1;
            if (!cached) {
                u.slots[1] = part_w1; u.tensor[1] = 1; u.fmt[1] = ssg::kE4M3;
                u.slots[2] = part_w2; u.tensor[2] = 2; u.fmt[2] = ssg::kE4M3;
                u.count = 3;
            }
            ssg::launch_scaling_update(state, u, st);
        }
        return check_launch("ssg_mlp_fwd");
    }

    // a5: factors s_i, s_i^-1 and the range of s^-1 * w3 (from the per-channel range of w3); plain block:
    // one scale for all of h, from its own range or as the caller gives it
    ssg::launch_channel_factors(h_camax, w3_camax, f, desc->smooth, s, sinv, scb + S_AMAX_W3S, scb + S_HMAX,
                                desc->h_scale_mode == SSG_SCALE_GIVEN ? desc->h_scale : nullptr, st);

    // a6: h^ = cast(s_i * h), recomputing h from the stored bf16 U, G
    ssg::CastArgs hq;
    hq.src = b + L.U; hq.src2 = b + L.G; hq.kind = ssg::SRC_SWIGLU; hq.rows = T; hq.cols = f; hq.fmt = ssg::kE4M3;
    hq.col_scale = s; hq.dst = b + L.h_q;
    hq.counters = reinterpret_cast<unsigned long long *>(desc->h_counters);

    // a7: w3~ = Q(s^-1 * w3); independent of a6, so the two share a launch
    ssg::CastArgs wq;
    wq.src = W3; wq.kind = ssg::SRC_BF16; wq.rows = dm; wq.cols = f; wq.fmt = ssg::kE4M3; wq.pow2 = pow2;
    wq.col_scale = sinv; wq.amax = sc + S_AMAX_W3S; wq.scale_out = sc + S_SW3;
    wq.dst = b + L.w3_q;
    if (gemm_grouping_enabled()) {
        ssg::launch_cast_h_w3(hq, wq, st);
    } else {
        ssg::launch_cast(hq, st);
        ssg::launch_cast(wq, st);
    }

    ssg::launch_gemm(g2, st);

    if (state) {
        // enter this call's ranges into the history; the scales written here serve the next call
        ssg::ScalingUpdate u;
        u.pow2 = pow2;
        u.slots[0] = delayed ? state_slots(0) : part_x; u.tensor[0] = 0; u.fmt[0] = ssg::kE4M3; u.count = 1;
        if (!cached) {
            u.slots[1] = delayed ? state_slots(1) : part_w1; u.tensor[1] = 1; u.fmt[1] = ssg::kE4M3;
            u.slots[2] = delayed ? state_slots(2) : part_w2; u.tensor[2] = 2; u.fmt[2] = ssg::kE4M3;
            u.count = 3;
        }
        ssg::launch_scaling_update(state, u, st);
    }
    return check_launch("ssg_mlp_fwd");
}

ssg_status ssg_mlp_bwd_plan(const ssg_mlp_desc *desc, int32_t compute_units, int32_t *dw3_sets_first,
                            int32_t *dw3_sets_total) {
    ssg_status rc = check_desc(desc, "ssg_mlp_bwd_plan");
    if (rc != SSG_OK) return rc;
    if (!dw3_sets_first || !dw3_sets_total) return fail(SSG_ERR_ARG, "ssg_mlp_bwd_plan: output pointers must not be NULL");
    if (compute_units <= 0 || compute_units > 4096)
        return fail(SSG_ERR_ARG, "ssg_mlp_bwd_plan: compute_units = %d (1 .. 4096)", (int)compute_units);
    BackwardGemms bg;
    backward_gemm_shapes(*desc, bg);
    const int all = ssg::gemm_tile_sets(bg.dw3);
    *dw3_sets_total = all;
    *dw3_sets_first = all;
    // the split exists only where both grouped launches are built: FP8 operands, the input gradient in one launch
    if (gemm_grouping_enabled() && !desc->w3_layer_bf16 && bg.dx.part == 3) {
        const ssg::GemmArgs *second[3] = {&bg.dx, &bg.dw1, &bg.dw2};
        *dw3_sets_first = ssg::gemm_group_split_sets(bg.dh, bg.dw3, second, 3, compute_units);
    }
    return SSG_OK;
}

ssg_status ssg_mlp_bwd(const ssg_mlp_desc *desc, const void *dy, const void *saved, size_t saved_bytes, void *dx,
                       void *dW1, void *dW2, void *dW3, void *workspace, size_t workspace_bytes, void *stream) {
    ssg_status rc = check_desc(desc, "ssg_mlp_bwd");
    if (rc != SSG_OK) return rc;
    SSG_REQUIRE_PTR(dy); SSG_REQUIRE_PTR(saved); SSG_REQUIRE_PTR(dx);
    SSG_REQUIRE_PTR(dW1); SSG_REQUIRE_PTR(dW2); SSG_REQUIRE_PTR(dW3); SSG_REQUIRE_PTR(workspace);
    hipStream_t st = (hipStream_t)stream;
    const int64_t T = desc->T, dm = desc->d, f = desc->f;
    const int pow2 = desc->rnd == SSG_ROUND_POW2;
    const SavedLayout L = saved_layout(*desc);
    const WorkLayout Wl = work_layout(*desc);
    if (saved_bytes < L.total)
        return fail(SSG_ERR_WORKSPACE, "ssg_mlp_bwd: saved holds %zu bytes, %zu needed (ssg_mlp_saved_bytes)", saved_bytes, L.total);
    if (workspace_bytes < Wl.total)
        return fail(SSG_ERR_WORKSPACE, "ssg_mlp_bwd: workspace holds %zu bytes, %zu needed (ssg_mlp_workspace_bytes)",
                    workspace_bytes, Wl.total);
    const uint8_t *sv = static_cast<const uint8_t *>(saved);
    uint8_t *wk = static_cast<uint8_t *>(workspace);
    const float *sc = reinterpret_cast<const float *>(sv + L.scalars);
    const float *s = reinterpret_cast<const float *>(sv + L.s), *sinv = reinterpret_cast<const float *>(sv + L.sinv);
    float *wsc = reinterpret_cast<float *>(wk + Wl.scalars);
    uint32_t *wscb = reinterpret_cast<uint32_t *>(wsc);
    const int dw_f32 = desc->dw_dtype == SSG_F32;

    uint32_t *wpart = reinterpret_cast<uint32_t *>(wk + Wl.partials);
    uint32_t *part_dy = wpart, *part_du = wpart + ssg::kAmaxSlotWords, *part_dg = wpart + 2 * ssg::kAmaxSlotWords;

    const bool delayed = desc->scale_mode == SSG_SCALE_DELAYED;
    uint32_t *state = static_cast<uint32_t *>(desc->scaling_state);
    auto state_scale = [&](int k) { return reinterpret_cast<float *>(state + (size_t)k * ssg::kScalingStride); };
    uint32_t *state_dy_slots = state ? state + ssg::kScalingHeaderWords + 3 * ssg::kAmaxSlotWords : nullptr;

    // every GEMM argument set is built and checked before the first launch: shapes, formats and layouts from
    // backward_gemm_shapes, operands, scales and results here
    BackwardGemms bg;
    backward_gemm_shapes(*desc, bg);
    const bool bf16_last = desc->w3_layer_bf16 != 0;
    // a10: dH; plain block: dH = acc / (sdy sw3), no channel factor
    ssg::GemmArgs &g = bg.dh;
    g.A = wk + Wl.dy_q; g.B = sv + L.w3_q; g.sa = wsc + W_SDY; g.sb = sc + S_SW3;
    g.col_scale = desc->smooth ? s : nullptr;
    g.U = sv + L.U; g.G = sv + L.G; g.C = wk + Wl.dU; g.C2 = wk + Wl.dG; g.amax_bits = part_du; g.amax_bits2 = part_dg;
    if (delayed && !bf16_last) {
        // the scales of dU, dG are known beforehand: the epilogue writes their E5M2 codes directly (a11 is fused
        // away; bf16 dU, dG are not stored) and still folds their ranges for the history
        g.C = wk + Wl.du_q; g.C2 = wk + Wl.dg_q;
        g.q_scale = state_scale(4); g.q_scale2 = state_scale(5); g.q_scale_out = wsc + W_SDU; g.q_scale_out2 = wsc + W_SDG;
        if (desc->keep_bf16_grads) { g.keep_u = wk + Wl.dU; g.keep_g = wk + Wl.dG; }
    }
    // a12: dW3 (plain: / (sdy * sigma_h))
    ssg::GemmArgs &g3 = bg.dw3;
    g3.A = wk + Wl.dy_q; g3.B = sv + L.h_q; g3.sa = wsc + W_SDY; g3.sb = desc->smooth ? nullptr : s;
    g3.col_scale = desc->smooth ? sinv : nullptr; g3.C = dW3;
    // a13: dX.  One launch that runs both products into the same accumulators where the shape allows (whole K steps
    // and tile columns); otherwise two launches, the first product through fp32 scratch
    float *dx_tmp = reinterpret_cast<float *>(wk + Wl.dx_tmp);
    ssg::GemmArgs &g4a = bg.dx;
    const bool dx_one = g4a.part == 3;
    g4a.A = wk + Wl.du_q; g4a.B = sv + L.w1_q; g4a.sa = wsc + W_SDU; g4a.sb = sc + S_SW1; g4a.C = dx_tmp;
    ssg::GemmArgs g4b = g4a;
    g4b.part = 2;
    g4b.A = wk + Wl.dg_q; g4b.B = sv + L.w2_q; g4b.sa = wsc + W_SDG; g4b.sb = sc + S_SW2; g4b.add = dx_tmp;
    g4b.C = dx; g4b.c_f32 = desc->y_dtype == SSG_F32;
    if (dx_one) {
        g4a.C = dx;
        g4a.A_ph2 = g4b.A; g4a.B_ph2 = g4b.B; g4a.sa_ph2 = g4b.sa; g4a.sb_ph2 = g4b.sb;
    }
    // a14: dW1, dW2
    ssg::GemmArgs &g5a = bg.dw1, &g5b = bg.dw2;
    g5a.A = wk + Wl.du_q; g5a.B = sv + L.x_q; g5a.sa = wsc + W_SDU; g5a.sb = sc + S_SX; g5a.C = dW1;
    g5b.A = wk + Wl.dg_q; g5b.B = sv + L.x_q; g5b.sa = wsc + W_SDG; g5b.sb = sc + S_SX; g5b.C = dW2;
    if (bf16_last) {
        // Section 4.3: dH = dY W3 and dW3 = dY^T h_b on bf16 operands (the transposed copies give every operand its
        // contraction index contiguous), no scales, no channel factors
        g.A = static_cast<const uint8_t *>(dy); g.B = sv + L.w3T; g.sa = nullptr; g.sb = nullptr; g.col_scale = nullptr;
        g3.A = wk + Wl.dyT; g3.B = sv + L.h_bT; g3.sa = nullptr; g3.sb = nullptr; g3.col_scale = nullptr;
    }
    for (const ssg::GemmArgs *a : {&g, &g3, &g4a, &g5a, &g5b})
        if (!ssg::gemm_args_ok(*a)) return fail(SSG_ERR_ARG, "ssg_mlp_bwd: internal GEMM arguments");
    if (!dx_one && !ssg::gemm_args_ok(g4b)) return fail(SSG_ERR_ARG, "ssg_mlp_bwd: internal GEMM arguments");
    // Grouped launches: {dH, dW3} (both read dY^; dW3 does not wait for dU, dG) and {dX, dW1, dW2} share one grid
    // each, so that a partly filled last round of workgroups is paid once per group and the epilogue traffic of one
    // GEMM runs under the main loops of the others
    const ssg::GemmArgs *group_a[2] = {&g, &g3}, *group_b[4] = {&g4a, &g5a, &g5b, &g3};
    const bool grouped_b = gemm_grouping_enabled() && dx_one && ssg::gemm_group_ok(group_b, 3);
    const bool grouped = grouped_b && ssg::gemm_group_ok(group_a, 2) && ssg::gemm_group_ok(group_b, 4);
    if ((rc = check_entry("ssg_mlp_bwd")) != SSG_OK) return rc;
    // dW3 depends only on dY^ and h^, so its tiles may run in either grouped launch: the first takes as many sets of
    // them as fill its last round, the second the rest
    const int dw3_sets = ssg::gemm_tile_sets(g3);
    const int dw3_split = grouped ? dw3_split_sets(g, g3, group_b) : dw3_sets;

    ssg::launch_fill_u32(wscb, (Wl.partials - Wl.scalars) / 4 + 3 * ssg::kAmaxSlotWords, 0u, st);

    // a9: upstream gradient to E5M2 (Section 6.2)
    ssg::CastArgs c;
    c.src = dy; c.kind = ssg::SRC_BF16; c.rows = T; c.cols = dm; c.fmt = ssg::kE5M2; c.pow2 = pow2;
    c.amax_slots = ssg::kAmaxSlots; c.scale_out = wsc + W_SDY; c.dst = wk + Wl.dy_q;
    if (bf16_last) {
        // dY is used as the bf16 tensor it is; only its transposed copy is needed (for dW3)
        ssg::launch_transpose_bf16(dy, T, dm, wk + Wl.dyT, st);
    } else if (delayed) {
        c.scale_in = state_scale(3); c.record = state_dy_slots;
    } else {
        ssg::launch_amax(dy, ssg::SRC_BF16, (size_t)(T * dm), part_dy, ssg::kAmaxSlots, st);
        c.amax = reinterpret_cast<float *>(part_dy); c.amax_out = wsc + W_AMAX_DY;
    }
    if (!bf16_last) ssg::launch_cast(c, st);
    c.record = nullptr;

    if (grouped) ssg::launch_gemm_group(group_a, 2, dw3_split, st);
    else ssg::launch_gemm(g, st);

    // a11: two tensors, two E5M2 scales (their ranges came out of the epilogue above either way), one launch
    if (!delayed) {                      // (under delayed scaling the epilogue above wrote the codes already)
        ssg::CastArgs gc[2];
        for (int k = 0; k < 2; ++k) {
            gc[k].kind = ssg::SRC_BF16; gc[k].fmt = ssg::kE5M2; gc[k].pow2 = pow2; gc[k].amax_slots = ssg::kAmaxSlots;
            gc[k].rows = T; gc[k].cols = f;
        }
        gc[0].src = wk + Wl.dU; gc[0].amax = reinterpret_cast<float *>(part_du); gc[0].amax_out = wsc + W_AMAX_DU;
        gc[0].scale_out = wsc + W_SDU; gc[0].dst = wk + Wl.du_q;
        gc[1].src = wk + Wl.dG; gc[1].amax = reinterpret_cast<float *>(part_dg); gc[1].amax_out = wsc + W_AMAX_DG;
        gc[1].scale_out = wsc + W_SDG; gc[1].dst = wk + Wl.dg_q;
        ssg::launch_cast_batch(gc, 2, st);
    }
    if (grouped) {
        if (dw3_split < dw3_sets) ssg::launch_gemm_group(group_b, 4, dw3_split, st);
        else ssg::launch_gemm_group(group_b, 3, -1, st);
    } else if (grouped_b) {
        ssg::launch_gemm(g3, st);
        ssg::launch_gemm_group(group_b, 3, -1, st);
    } else {
        ssg::launch_gemm(g3, st);
        ssg::launch_gemm(g4a, st);
        if (!dx_one) ssg::launch_gemm(g4b, st);
        ssg::launch_gemm(g5a, st);
        ssg::launch_gemm(g5b, st);
    }
    if (state) {
        ssg::ScalingUpdate u;
        u.pow2 = pow2; u.count = 3;
        u.slots[0] = delayed ? state_dy_slots : part_dy; u.tensor[0] = 3; u.fmt[0] = ssg::kE5M2;
        u.slots[1] = part_du; u.tensor[1] = 4; u.fmt[1] = ssg::kE5M2;
        u.slots[2] = part_dg; u.tensor[2] = 5; u.fmt[2] = ssg::kE5M2;
        if (bf16_last) {                 // dY is not quantized: no range of it was taken
            u.slots[0] = part_du; u.tensor[0] = 4; u.slots[1] = part_dg; u.tensor[1] = 5; u.count = 2;
        }
        ssg::launch_scaling_update(state, u, st);
    }
    return check_launch("ssg_mlp_bwd");
}

}  // extern "C"
