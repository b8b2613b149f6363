// C ABI of libvatp: argument checks, workspace carving and kernel dispatch.
// Declarations and the contract of every call are in include/vatp.h.
#include <math.h>
#include <string.h>
#include <new>

#include "vatp_device.h"

using namespace vatp;

struct vatp_ctx {
    int device;
    void *scratch;       // this device's copy of the static scratch array (address looked up at creation)
};

// Scratch memory of vatp_decode_prune_step_static, the entry point for callers that cannot allocate: a
// file-scope device array, so every GPU the library runs on holds VATP_STATIC_SCRATCH_BYTES of it until the
// process ends.  In host code the name is only a handle: the address on a device comes from
// hipGetSymbolAddress (vatp_create, with that device current), and only that address is ever used.
static __device__ __align__(256) unsigned char scratch[VATP_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Prepared {
    BatchMeta meta;
    Geometry g;
};

vatp_status check_params(const vatp_params *p, int which_call)
{
    if (!p || !p->len) return VATP_E_NULL;
    const bool prunes = which_call == VATP_CALL_SELECT_COMPACT || which_call == VATP_CALL_DECODE_PRUNE_STEP;
    const bool decodes = which_call == VATP_CALL_DECODE_STEP || which_call == VATP_CALL_DECODE_ATTEND_STEP ||
                         which_call == VATP_CALL_DECODE_PRUNE_STEP;
    if (prunes && !p->budget) return VATP_E_NULL;
    if (which_call < VATP_CALL_PREFILL_SCORE || which_call > VATP_CALL_PREFILL_SCORE_WINDOW) return VATP_E_SHAPE;
    if (p->dtype != VATP_F32 && p->dtype != VATP_BF16) return VATP_E_DTYPE;
    if (p->batch < 1 || p->batch > VATP_MAX_BATCH || p->n_heads < 1) return VATP_E_SHAPE;
    if (p->q_per_kv < 0 || p->q_per_kv > VATP_MAX_GROUP) return VATP_E_SHAPE;
    const int group = p->q_per_kv > 1 ? p->q_per_kv : 1;
    if (static_cast<int64_t>(p->batch) * p->n_heads * group > VATP_MAX_UNITS) return VATP_E_SHAPE;
    if (p->head_dim != 64 && p->head_dim != 128) return VATP_E_SHAPE;
    if (p->cap < 1 || p->cap_out < 0 || p->n_sink < 0 || p->recent < 0) return VATP_E_SHAPE;
    if (p->cap > VATP_MAX_CAP || p->cap_out > VATP_MAX_CAP) return VATP_E_SHAPE;   // 32-bit byte offsets inside a unit
    if (!(p->scale >= 0.f) || isinf(p->scale)) return VATP_E_SHAPE;
    if (p->norm < VATP_NORM_L1 || p->norm > VATP_NORM_NONE) return VATP_E_SHAPE;
    // element counts of one buffer stay below 2^40 (indexing is 64-bit, row indices 32-bit)
    if (static_cast<double>(p->batch) * p->n_heads * static_cast<double>(p->cap > p->cap_out ? p->cap : p->cap_out) *
            p->head_dim > 1099511627776.0)
        return VATP_E_SHAPE;
    const int cap_out = p->cap_out ? p->cap_out : p->cap;
    for (int b = 0; b < p->batch; ++b) {
        const int len = p->len[b];
        if (len < 0 || len > p->cap) return VATP_E_SHAPE;
        if (decodes && len + 1 > p->cap) return VATP_E_SHAPE;
        if (prunes) {
            const int B = p->budget[b];
            const int n = decodes ? len + 1 : len;         // rows the selection sees
            if (B < 0 || B < p->n_sink + p->recent) return VATP_E_BUDGET;
            const int n_keep = n < B ? n : B;
            if (n_keep > cap_out) return VATP_E_BUDGET;
            if (decodes && n > B + 1) return VATP_E_BUDGET;    // the fused step removes one row at most
        }
    }
    return VATP_OK;
}

void prepare(const vatp_params *p, int which_call, const int32_t *new_pos, Prepared *out)
{
    Geometry &g = out->g;
    g.batch = p->batch;
    g.n_heads = p->n_heads;
    g.cap = p->cap;
    g.cap_out = p->cap_out ? p->cap_out : p->cap;
    g.n_sink = p->n_sink;
    g.recent = p->recent;
    g.norm = p->norm;
    g.group = p->q_per_kv > 1 ? p->q_per_kv : 1;
    const double c = p->scale > 0.f ? static_cast<double>(p->scale) : 1.0 / sqrt(static_cast<double>(p->head_dim));
    g.scale_log2 = static_cast<float>(c * 1.4426950408889634074);
    g.max_len = 0;
    g.stream = 0;
    memset(&out->meta, 0, sizeof(out->meta));
    for (int b = 0; b < p->batch; ++b) {
        const int len = p->len[b];
        out->meta.len[b] = len;
        int extent = len;
        if (which_call == VATP_CALL_DECODE_STEP || which_call == VATP_CALL_DECODE_ATTEND_STEP ||
            which_call == VATP_CALL_DECODE_PRUNE_STEP) {
            out->meta.aux[b] = new_pos ? new_pos[b] : 0;
            extent = len + 1;
        } else if (which_call == VATP_CALL_SELECT_COMPACT) {
            out->meta.aux[b] = p->budget[b];
            extent = len < p->budget[b] ? len : p->budget[b];
        }
        if (extent > g.max_len) g.max_len = extent;
    }
    // streaming (non-temporal) accesses when the cache rows this call may touch will not stay resident anyway
    size_t rows = 0;
    for (int b = 0; b < p->batch; ++b) rows += static_cast<size_t>(p->len[b] > 0 ? p->len[b] : 0);
    g.stream = stream_rows(static_cast<size_t>(p->n_heads), rows, static_cast<size_t>(p->head_dim) * (p->dtype == VATP_BF16 ? 2 : 4));
}

// the context's device must be the current one: kernels are launched on the current device
inline bool wrong_device(const vatp_ctx *ctx)
{
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) {
        (void)hipGetLastError();
        return true;
    }
    return cur != ctx->device;
}

inline bool misaligned(const void *ptr, size_t a) { return (reinterpret_cast<uintptr_t>(ptr) & (a - 1)) != 0; }

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char *vatp_strerror(vatp_status st)
{
    switch (st) {
    case VATP_OK: return "ok";
    case VATP_E_NULL: return "a required pointer is NULL";
    case VATP_E_SHAPE: return "shape out of range (batch, heads, head_dim, cap or len)";
    case VATP_E_DTYPE: return "unsupported dtype";
    case VATP_E_BUDGET: return "budget smaller than n_sink + recent, larger than cap_out, or exceeded by more than one row in the fused step";
    case VATP_E_WORKSPACE: return "workspace missing, too small or misaligned";
    case VATP_E_DEVICE: return "HIP error";
    }
    return "unknown status";
}

vatp_status vatp_create(vatp_ctx **ctx, int device)
{
    if (!ctx) return VATP_E_NULL;
    *ctx = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) {
        (void)hipGetLastError();
        return VATP_E_DEVICE;
    }
    // the static scratch array's address on this device, looked up with the device current
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) {
        (void)hipGetLastError();
        return VATP_E_DEVICE;
    }
    if (prev != device && hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return VATP_E_DEVICE;
    }
    void *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (prev != device) (void)hipSetDevice(prev);
    if (e != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return VATP_E_DEVICE;
    }
    vatp_ctx *c = new (std::nothrow) vatp_ctx;
    if (!c) return VATP_E_DEVICE;
    c->device = device;
    c->scratch = ptr;
    *ctx = c;
    return VATP_OK;
}

void vatp_destroy(vatp_ctx *ctx)
{
    if (!ctx) return;
    delete ctx;
}

vatp_status vatp_validate(const vatp_params *p, int which_call) { return check_params(p, which_call); }

size_t vatp_workspace_bytes(const vatp_ctx *, const vatp_params *p, int which_call)
{
    if (check_params(p, which_call) != VATP_OK) return 0;
    // everything kept in the workspace is per query head
    const size_t units = static_cast<size_t>(p->batch) * p->n_heads * (p->q_per_kv > 1 ? p->q_per_kv : 1);
    switch (which_call) {
    case VATP_CALL_PREFILL_SCORE:           // lse2[units, cap] (+ as much again for partial column sums of a group)
        return align_up(units * p->cap * sizeof(float)) * (p->q_per_kv > 1 ? 2 : 1);
    case VATP_CALL_PREFILL_SCORE_WINDOW:    // ... + partial row statistics per range of keys
        return align_up(units * p->cap * sizeof(float)) +
               align_up(static_cast<size_t>(prefill_window_splits(p->cap)) * units * p->cap * sizeof(float));
    case VATP_CALL_DECODE_STEP: {           // logits[units, cap] + per-chunk softmax statistics
        const size_t chunks = (static_cast<size_t>(p->cap) + kDecodeChunk - 1) / kDecodeChunk;
        return align_up(units * p->cap * sizeof(float)) + align_up(units * chunks * sizeof(float2));
    }
    case VATP_CALL_DECODE_PRUNE_STEP:
    case VATP_CALL_DECODE_ATTEND_STEP: {    // ... + per-chunk partial attention outputs [units, chunks, d]
        const size_t chunks = (static_cast<size_t>(p->cap) + kDecodeChunk - 1) / kDecodeChunk;
        return align_up(units * p->cap * sizeof(float)) + align_up(units * chunks * sizeof(float2)) +
               align_up(units * chunks * p->head_dim * sizeof(float));
    }
    default:
        return 0;
    }
}

}  // extern "C" (reopened below)

namespace {

constexpr int kMaxWindow = 1 << 18;      // (the history gather indexes ring rows / 8 with a 16-bit grid dimension)

vatp_status prefill_score_impl(vatp_ctx *ctx, const vatp_params *p, const void *Q, const void *K, const void *V,
                               const float *lse, bool have_lse, int window, float *hist, float *S, float *nrm,
                               void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!ctx || !Q || !K || !V || !S || !nrm || (have_lse && !lse)) return VATP_E_NULL;
    if (window < -1 || window > kMaxWindow) return VATP_E_SHAPE;
    const vatp_status st = check_params(p, window < 0 ? VATP_CALL_PREFILL_SCORE : VATP_CALL_PREFILL_SCORE_WINDOW);
    if (st != VATP_OK) return st;
    if (wrong_device(ctx)) return VATP_E_DEVICE;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(hist, 4)) return VATP_E_SHAPE;
    const size_t need = vatp_workspace_bytes(ctx, p, window < 0 ? VATP_CALL_PREFILL_SCORE : VATP_CALL_PREFILL_SCORE_WINDOW);
    if (!ws || ws_bytes < need || misaligned(ws, kAlign)) return VATP_E_WORKSPACE;
    Prepared pr;
    prepare(p, VATP_CALL_PREFILL_SCORE, nullptr, &pr);
    const size_t units = static_cast<size_t>(p->batch) * p->n_heads;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float *lse2 = static_cast<float *>(ws);
    if (have_lse && launch_lse_to_base2(lse, lse2, pr.meta, pr.g, stream) != hipSuccess) return VATP_E_DEVICE;
    // bf16 with head_dim 128 runs on the matrix cores; everything else, and the history-window scores
    // (a band of w+1 query rows, a fraction of the full pass), on the fp32 FMA kernels
    const bool mfma = p->dtype == VATP_BF16 && p->head_dim == 128;
    hipError_t e;
    if (mfma && window < 0) {                 // (the matrix-core column-sum pass writes the norms as well)
        float *s_part = pr.g.group > 1 ? lse2 + align_up(units * pr.g.group * p->cap * sizeof(float)) / sizeof(float) : nullptr;
        e = launch_prefill_mfma(Q, K, V, S, nrm, lse2, s_part, have_lse, pr.meta, pr.g, stream);
    } else if (mfma && prefill_mfma_window_fits(window, p->cap, static_cast<int>(units * pr.g.group))) {
        e = launch_prefill_mfma_window(Q, K, V, S, nrm, lse2,
                                       lse2 + align_up(units * pr.g.group * p->cap * sizeof(float)) / sizeof(float), window,
                                       hist, pr.meta, pr.g, stream);
    } else {
        if (launch_l1norm(p->dtype, p->head_dim, V, nrm, pr.meta, pr.g, stream) != hipSuccess) return VATP_E_DEVICE;
        e = launch_prefill_generic(p->dtype, p->head_dim, Q, K, S, lse2, have_lse, window, hist, pr.meta, pr.g, stream);
    }
    if (e != hipSuccess) return VATP_E_DEVICE;
    return VATP_OK;
}

}  // namespace

extern "C" {

vatp_status vatp_prefill_score(vatp_ctx *ctx, const vatp_params *p, const void *Q, const void *K,
                               const void *V, float *S, float *nrm, void *ws, size_t ws_bytes,
                               void *hip_stream)
{
    return prefill_score_impl(ctx, p, Q, K, V, nullptr, false, -1, nullptr, S, nrm, ws, ws_bytes, hip_stream);
}

vatp_status vatp_prefill_score_window(vatp_ctx *ctx, const vatp_params *p, const void *Q, const void *K,
                                      const void *V, int32_t window, float *S, float *nrm, float *hist, void *ws,
                                      size_t ws_bytes, void *hip_stream)
{
    if (window < 0) return VATP_E_SHAPE;
    return prefill_score_impl(ctx, p, Q, K, V, nullptr, false, window, hist, S, nrm, ws, ws_bytes, hip_stream);
}

vatp_status vatp_prefill_score_lse(vatp_ctx *ctx, const vatp_params *p, const void *Q, const void *K,
                                   const void *V, const float *lse, float *S, float *nrm, void *ws,
                                   size_t ws_bytes, void *hip_stream)
{
    return prefill_score_impl(ctx, p, Q, K, V, lse, true, -1, nullptr, S, nrm, ws, ws_bytes, hip_stream);
}

}  // extern "C" (reopened below)

namespace {

vatp_status decode_step_impl(vatp_ctx *ctx, const vatp_params *p, int which_call, const void *q, const void *k,
                             const void *v, void *K, void *V, float *S, float *nrm, int32_t *pos,
                             const int32_t *new_pos, float *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!ctx || !q || !k || !v || !K || !V || !S || !nrm) return VATP_E_NULL;
    if (which_call == VATP_CALL_DECODE_ATTEND_STEP && !out) return VATP_E_NULL;
    if (pos && !new_pos) return VATP_E_NULL;
    const vatp_status st = check_params(p, which_call);
    if (st != VATP_OK) return st;
    if (wrong_device(ctx)) return VATP_E_DEVICE;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(K, 16) || misaligned(V, 16))
        return VATP_E_SHAPE;
    const size_t need = vatp_workspace_bytes(ctx, p, which_call);
    if (!ws || ws_bytes < need || misaligned(ws, kAlign)) return VATP_E_WORKSPACE;
    Prepared pr;
    prepare(p, which_call, pos ? new_pos : nullptr, &pr);
    const size_t units = static_cast<size_t>(p->batch) * p->n_heads * pr.g.group;      // query heads
    const size_t chunks = (static_cast<size_t>(p->cap) + kDecodeChunk - 1) / kDecodeChunk;
    char *base = static_cast<char *>(ws);
    float *ws_logit = reinterpret_cast<float *>(base);
    float2 *ws_part = reinterpret_cast<float2 *>(base + align_up(units * p->cap * sizeof(float)));
    float *ws_out = reinterpret_cast<float *>(base + align_up(units * p->cap * sizeof(float)) +
                                              align_up(units * chunks * sizeof(float2)));
    if (launch_decode(p->dtype, p->head_dim, q, k, v, K, V, S, nrm, pos, ws_logit, ws_part, out ? ws_out : nullptr,
                      out, true, pr.meta, pr.g, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return VATP_E_DEVICE;
    return VATP_OK;
}

}  // namespace

extern "C" {

vatp_status vatp_decode_step(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k,
                             const void *v, void *K, void *V, float *S, float *nrm, int32_t *pos,
                             const int32_t *new_pos, void *ws, size_t ws_bytes, void *hip_stream)
{
    return decode_step_impl(ctx, p, VATP_CALL_DECODE_STEP, q, k, v, K, V, S, nrm, pos, new_pos, nullptr, ws, ws_bytes,
                            hip_stream);
}

vatp_status vatp_decode_attend_step(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k,
                                    const void *v, void *K, void *V, float *S, float *nrm, int32_t *pos,
                                    const int32_t *new_pos, float *out, void *ws, size_t ws_bytes,
                                    void *hip_stream)
{
    return decode_step_impl(ctx, p, VATP_CALL_DECODE_ATTEND_STEP, q, k, v, K, V, S, nrm, pos, new_pos, out, ws,
                            ws_bytes, hip_stream);
}

}  // extern "C" (reopened below)

namespace {

vatp_status decode_prune_impl(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k, const void *v,
                              void *K, void *V, const float *S, float *nrm, int32_t *pos, const int32_t *new_pos,
                              void *K_out, void *V_out, float *S_out, float *nrm_out, int32_t *pos_out,
                              int32_t *kept_idx, const int32_t *synced_in, int32_t *synced_out, WindowArgs &win,
                              float *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!ctx || !q || !k || !v || !K || !V || !S || !nrm || !K_out || !V_out || !S_out || !nrm_out || !synced_in ||
        !synced_out)
        return VATP_E_NULL;
    if ((pos == nullptr) != (pos_out == nullptr) || (pos && !new_pos)) return VATP_E_NULL;
    const vatp_status st = check_params(p, VATP_CALL_DECODE_PRUNE_STEP);
    if (st != VATP_OK) return st;
    if (wrong_device(ctx)) return VATP_E_DEVICE;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(K, 16) || misaligned(V, 16) ||
        misaligned(K_out, 16) || misaligned(V_out, 16))
        return VATP_E_SHAPE;
    if (K_out == K || V_out == V || S_out == S || nrm_out == nrm || (pos && pos_out == pos) || synced_in == synced_out)
        return VATP_E_SHAPE;
    const size_t need = vatp_workspace_bytes(ctx, p, VATP_CALL_DECODE_PRUNE_STEP);
    if (!ws || ws_bytes < need || misaligned(ws, kAlign)) return VATP_E_WORKSPACE;
    Prepared pr;
    prepare(p, VATP_CALL_DECODE_PRUNE_STEP, pos ? new_pos : nullptr, &pr);
    const size_t kv_units = static_cast<size_t>(p->batch) * p->n_heads;
    const size_t units = kv_units * pr.g.group;                               // query heads
    const size_t chunks = (static_cast<size_t>(p->cap) + kDecodeChunk - 1) / kDecodeChunk;
    char *base = static_cast<char *>(ws);
    float *ws_logit = reinterpret_cast<float *>(base);
    float2 *ws_part = reinterpret_cast<float2 *>(base + align_up(units * p->cap * sizeof(float)));
    float *ws_out = reinterpret_cast<float *>(base + align_up(units * p->cap * sizeof(float)) +
                                              align_up(units * chunks * sizeof(float2)));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    BatchMeta budgets = pr.meta;
    for (int b = 0; b < p->batch; ++b) budgets.aux[b] = p->budget[b];
    // One launch with a workgroup per head when there are enough heads to fill the chip that way and
    // each is short enough for a single workgroup to stream quickly (measured per step at 256 heads x 820 rows:
    // 22 against 30 us with 32 layers' caches in turn; slower than two launches
    // at 32 heads x 2049 rows, 23 against 14 us).
    const bool one = !out && !win.hist && pr.g.group == 1 && kv_units >= 128 && pr.g.max_len <= 1024 &&
                     pr.g.max_len <= decode_prune_one_max_rows();
    if (one) {
        BudgetList blist;
        memcpy(blist.v, budgets.aux, sizeof(blist.v));
        if (launch_decode_prune_one(p->dtype, p->head_dim, q, k, v, K, V, S, nrm, pos, K_out, V_out, S_out, nrm_out,
                                    pos_out, kept_idx, synced_in, synced_out, pr.meta, blist, pr.g, stream) !=
            hipSuccess)
            return VATP_E_DEVICE;
        return VATP_OK;
    }
    // first launch: append the row, logits and chunk statistics (S is not touched)
    if (launch_decode(p->dtype, p->head_dim, q, k, v, K, V, nullptr, nrm, pos, ws_logit, ws_part,
                      out ? ws_out : nullptr, out, false, pr.meta, pr.g, stream) != hipSuccess)
        return VATP_E_DEVICE;
    // second launch: new scores, the evicted row, the out-of-date rows of the other set
    if (launch_decode_prune(p->dtype, p->head_dim, K, V, S, nrm, pos, K_out, V_out, S_out, nrm_out, pos_out, kept_idx,
                            synced_in, synced_out, ws_logit, ws_part, out ? ws_out : nullptr, out, win, budgets,
                            pr.g, stream) != hipSuccess)
        return VATP_E_DEVICE;
    return VATP_OK;
}

}  // namespace

extern "C" {

vatp_status vatp_decode_prune_step(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k,
                                   const void *v, void *K, void *V, const float *S, float *nrm, int32_t *pos,
                                   const int32_t *new_pos, void *K_out, void *V_out, float *S_out,
                                   float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                                   const int32_t *synced_in, int32_t *synced_out, float *out, void *ws,
                                   size_t ws_bytes, void *hip_stream)
{
    WindowArgs win = {};
    return decode_prune_impl(ctx, p, q, k, v, K, V, S, nrm, pos, new_pos, K_out, V_out, S_out, nrm_out, pos_out,
                             kept_idx, synced_in, synced_out, win, out, ws, ws_bytes, hip_stream);
}

vatp_status vatp_decode_prune_step_static(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k,
                                          const void *v, void *K, void *V, const float *S, float *nrm, int32_t *pos,
                                          const int32_t *new_pos, void *K_out, void *V_out, float *S_out,
                                          float *nrm_out, int32_t *pos_out, int32_t *kept_idx,
                                          const int32_t *synced_in, int32_t *synced_out, float *out,
                                          void *hip_stream)
{
    if (!ctx) return VATP_E_NULL;
    const vatp_status st = check_params(p, VATP_CALL_DECODE_PRUNE_STEP);
    if (st != VATP_OK) return st;
    // the step's workspace is the device's static array: nothing is allocated, sizes beyond it are refused
    const size_t need = vatp_workspace_bytes(ctx, p, VATP_CALL_DECODE_PRUNE_STEP);
    if (need > static_cast<size_t>(VATP_STATIC_SCRATCH_BYTES)) return VATP_E_WORKSPACE;
    WindowArgs win = {};
    return decode_prune_impl(ctx, p, q, k, v, K, V, S, nrm, pos, new_pos, K_out, V_out, S_out, nrm_out, pos_out,
                             kept_idx, synced_in, synced_out, win, out, ctx->scratch, VATP_STATIC_SCRATCH_BYTES,
                             hip_stream);
}

vatp_status vatp_decode_prune_step_window(vatp_ctx *ctx, const vatp_params *p, const void *q, const void *k,
                                          const void *v, void *K, void *V, const float *S, float *nrm,
                                          int32_t *pos, int32_t *hid, const int32_t *new_pos, void *K_out,
                                          void *V_out, float *S_out, float *nrm_out, int32_t *pos_out,
                                          int32_t *hid_out, int32_t *kept_idx, const int32_t *synced_in,
                                          int32_t *synced_out, const int32_t *free_in, int32_t *free_out,
                                          float *hist, const float *S_lo, float *S_lo_out, int32_t window,
                                          int32_t cap_hist, float *out, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!p || !hid || !hid_out || !free_in || !free_out || !hist || !new_pos || !S_lo || !S_lo_out) return VATP_E_NULL;
    if (window < 0 || window > kMaxWindow || hid == hid_out || free_in == free_out || S_lo == S_lo_out)
        return VATP_E_SHAPE;
    if (p->batch < 1 || p->batch > VATP_MAX_BATCH || !p->budget) return p->budget ? VATP_E_SHAPE : VATP_E_NULL;
    WindowArgs win = {};
    win.hist = hist;
    win.s_lo = S_lo;
    win.s_lo_out = S_lo_out;
    win.hid = hid;
    win.hid_out = hid_out;
    win.free_in = free_in;
    win.free_out = free_out;
    win.rows = window + 2;
    win.cap_hist = cap_hist;
    for (int b = 0; b < p->batch; ++b) {
        if (new_pos[b] < 0) return VATP_E_SHAPE;
        if (cap_hist < p->budget[b] + 1) return VATP_E_BUDGET;        // one column per row plus the appended one
        win.step[b] = new_pos[b];
    }
    return decode_prune_impl(ctx, p, q, k, v, K, V, S, nrm, pos, new_pos, K_out, V_out, S_out, nrm_out, pos_out,
                             kept_idx, synced_in, synced_out, win, out, ws, ws_bytes, hip_stream);
}

vatp_status vatp_select_compact_window(vatp_ctx *ctx, const vatp_params *p, const void *K, const void *V,
                                       const float *S, const float *nrm, const int32_t *pos, const float *hist,
                                       int32_t window, void *K_out, void *V_out, float *S_out, float *nrm_out,
                                       int32_t *pos_out, int32_t *kept_idx, float *hist_out, int32_t cap_hist,
                                       int32_t *hid_out, int32_t *free_out, float *S_lo_out, void *ws,
                                       size_t ws_bytes, void *hip_stream)
{
    if (!hist || !hist_out || !hid_out || !free_out || !S_lo_out) return VATP_E_NULL;
    if (window < 0 || window > kMaxWindow || hist == hist_out) return VATP_E_SHAPE;
    vatp_status st = check_params(p, VATP_CALL_SELECT_COMPACT);
    if (st != VATP_OK) return st;
    for (int b = 0; b < p->batch; ++b)
        if (cap_hist < (p->len[b] < p->budget[b] ? p->len[b] : p->budget[b])) return VATP_E_BUDGET;
    st = vatp_select_compact(ctx, p, K, V, S, nrm, pos, K_out, V_out, S_out, nrm_out, pos_out, kept_idx, ws, ws_bytes,
                             hip_stream);
    if (st != VATP_OK) return st;
    Prepared pr;
    prepare(p, VATP_CALL_SELECT_COMPACT, nullptr, &pr);
    if (launch_hist_gather(hist, kept_idx, hist_out, hid_out, free_out, S_out, S_lo_out, window + 2, cap_hist, pr.meta, pr.g,
                           static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return VATP_E_DEVICE;
    return VATP_OK;
}

vatp_status vatp_select_compact(vatp_ctx *ctx, const vatp_params *p, const void *K, const void *V,
                                const float *S, const float *nrm, const int32_t *pos, void *K_out,
                                void *V_out, float *S_out, float *nrm_out, int32_t *pos_out,
                                int32_t *kept_idx, void *, size_t, void *hip_stream)
{
    if (!ctx || !K || !V || !S || !nrm || !K_out || !V_out || !S_out || !nrm_out || !kept_idx) return VATP_E_NULL;
    if ((pos == nullptr) != (pos_out == nullptr)) return VATP_E_NULL;
    const vatp_status st = check_params(p, VATP_CALL_SELECT_COMPACT);
    if (st != VATP_OK) return st;
    if (wrong_device(ctx)) return VATP_E_DEVICE;
    if (misaligned(K, 16) || misaligned(V, 16) || misaligned(K_out, 16) || misaligned(V_out, 16)) return VATP_E_SHAPE;
    if (K_out == K || V_out == V || S_out == S || nrm_out == nrm || (pos && pos_out == pos)) return VATP_E_SHAPE;
    Prepared pr;
    prepare(p, VATP_CALL_SELECT_COMPACT, nullptr, &pr);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    bool evict_one = true;            // every sequence loses at most one row
    for (int b = 0; b < p->batch; ++b)
        if (p->len[b] > p->budget[b] + 1) evict_one = false;
    if (!evict_one) {
        if (launch_select(S, nrm, kept_idx, pr.meta, pr.g, stream) != hipSuccess) return VATP_E_DEVICE;
    }
    if (launch_gather(p->dtype, p->head_dim, evict_one, K, V, S, nrm, pos, K_out, V_out, S_out, nrm_out, pos_out,
                      kept_idx, pr.meta, pr.g, stream) != hipSuccess)
        return VATP_E_DEVICE;
    return VATP_OK;
}

}  // extern "C"
#pragma GCC visibility pop
