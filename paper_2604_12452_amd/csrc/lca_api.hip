// C ABI of liblca: argument validation, workspace carving and kernel dispatch.  No allocation, no
// synchronisation, no state beyond the thread-local error string, the device array of lca_condense_noalloc
// and its per-device address.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "lca_internal.h"

namespace {

thread_local char g_err[512] = "";

lca_status fail(lca_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validate the descriptor and derive sizes. `decode`: L counts the token being decoded.
lca_status make_dims(const lca_desc *desc, lca::Dims &d)
{
    if (desc == nullptr) return fail(LCA_ERR_INVALID_ARG, "desc is NULL");
    if (desc->B <= 0 || desc->L <= 0 || desc->H <= 0 || desc->S <= 0) return fail(LCA_ERR_INVALID_ARG, "B, L, H, S must be positive");
    if (desc->H % desc->S != 0) return fail(LCA_ERR_INVALID_ARG, "H (%d) must be a multiple of S (%d)", desc->H, desc->S);
    if (desc->g <= 0 || desc->g > 64) return fail(LCA_ERR_INVALID_ARG, "g must be in [1, 64], got %d", desc->g);
    if (desc->w < 0) return fail(LCA_ERR_INVALID_ARG, "w must be >= 0");
    if (desc->mode != LCA_MODE_MLA && desc->mode != LCA_MODE_GQA) return fail(LCA_ERR_INVALID_ARG, "unknown mode %d", desc->mode);
    if (desc->dtype != LCA_BF16 && desc->dtype != LCA_F32 && desc->dtype != LCA_F16) return fail(LCA_ERR_INVALID_ARG, "unknown dtype %d", desc->dtype);
    const int mult = desc->dtype == LCA_F32 ? 4 : 8;
    if (desc->d_pool <= 0 || desc->d_sel <= 0 || desc->d_pool % mult || desc->d_sel % mult)
        return fail(LCA_ERR_INVALID_ARG, "d_pool and d_sel must be positive multiples of %d", mult);
    const int d_qk = desc->mode == LCA_MODE_MLA ? desc->d_pool + desc->d_sel : desc->d_sel;
    if (d_qk > 1024 || desc->d_pool > 1024) return fail(LCA_ERR_UNSUPPORTED, "d_qk and d_pool above 1024 are not supported");
    const int n_q = desc->n_q == 0 ? desc->g : desc->n_q;
    if (n_q < 0) return fail(LCA_ERR_INVALID_ARG, "n_q (%d) must not be negative", n_q);
    if (!(desc->scale == desc->scale) || !(desc->rep_logit_bias == desc->rep_logit_bias)) return fail(LCA_ERR_INVALID_ARG, "scale / bias is NaN");
    if ((long long)desc->B * desc->L * desc->H >= (1ll << 31)) return fail(LCA_ERR_UNSUPPORTED, "B*L*H must be below 2^31");
    d.B = desc->B; d.L = desc->L; d.H = desc->H; d.S = desc->S;
    d.P = desc->mode == LCA_MODE_MLA ? 1 : desc->S;
    d.d_pool = desc->d_pool; d.d_sel = desc->d_sel; d.d_qk = d_qk; d.d_v = desc->d_pool;
    d.g = desc->g; d.w = desc->w; d.n_q = n_q;
    d.m = desc->L > desc->w ? (desc->L - desc->w) / desc->g : 0;
    d.k = desc->L - d.m * desc->g;
    d.mode = desc->mode; d.dtype = desc->dtype; d.elt = desc->dtype == LCA_F32 ? 4 : 2;
    d.scale = desc->scale; d.rep_logit_bias = desc->rep_logit_bias;
    if (desc->pool_reduce < 0 || desc->pool_reduce > LCA_REDUCE_MAXPOOL || desc->sel_reduce < 0 || desc->sel_reduce > LCA_REDUCE_MAXPOOL)
        return fail(LCA_ERR_INVALID_ARG, "unknown reduce strategy (%d, %d)", desc->pool_reduce, desc->sel_reduce);
    d.pool_reduce = desc->pool_reduce == LCA_REDUCE_DEFAULT ? LCA_REDUCE_WEIGHTED : desc->pool_reduce;
    d.sel_reduce = desc->sel_reduce == LCA_REDUCE_DEFAULT ? LCA_REDUCE_MAXSEL : desc->sel_reduce;
    return LCA_OK;
}

size_t qbar_bytes(const lca::Dims &d) { return (((size_t)d.B * d.S * d.d_qk * sizeof(float)) + 255) & ~(size_t)255; }

size_t workspace_bytes(const lca::Dims &d)
{
    size_t need = qbar_bytes(d);
    const size_t dec = lca::decode_workspace_bytes(d), dev = lca::deviation_workspace_bytes(d), up = lca::attn_mla_up_workspace_bytes(d);
    need = need > dec ? need : dec;
    need = need > up ? need : up;
    return need > dev ? need : dev;
}

lca_status check_ptr(const void *p, const char *name, bool required = true)
{
    if (p == nullptr) return required ? fail(LCA_ERR_INVALID_ARG, "%s is NULL", name) : LCA_OK;
    if (!aligned16(p)) return fail(LCA_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    return LCA_OK;
}

#define LCA_TRY(expr)                      \
    do {                                   \
        lca_status _s = (expr);            \
        if (_s != LCA_OK) return _s;       \
    } while (0)

lca_status check_ws(const lca::Dims &d, const void *ws, size_t ws_bytes)
{
    const size_t need = workspace_bytes(d);
    if (need == 0) return LCA_OK;
    if (ws == nullptr) return fail(LCA_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
    if (!aligned16(ws)) return fail(LCA_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    if (ws_bytes < need) return fail(LCA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return LCA_OK;
}

lca_status hip_status(hipError_t e, const char *what)
{
    if (e == hipSuccess) return LCA_OK;
    return fail(LCA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// The launch functions report hipGetLastError() after their kernels, and that call returns the calling thread's last
// error whoever caused it: one left behind by an earlier runtime call of the caller's own would be taken for a failed
// launch.  So the thread's error state is read, and thereby cleared, right before a launch function runs.
#define LCA_LAUNCH(call, what) ((void)hipGetLastError(), hip_status((call), (what)))

// The two matrix-core kernels take their widths in a 16-bit type with a positive scale (their fixed-reference softmax
// orders logits by the raw products); every other descriptor, a zero or negative scale included, runs the general kernel.
lca_status run_attn(const lca::AttnArgs &a, hipStream_t st, const char *what)
{
    if (lca::attn_mla_supported(a.d)) return LCA_LAUNCH(lca::launch_attn_mla(a, st), what);
    if (lca::attn_gqa64_supported(a.d)) return LCA_LAUNCH(lca::launch_attn_gqa64(a, st), what);
    return LCA_LAUNCH(lca::launch_attn_simple(a, st), what);
}

// ---- lca_condense_noalloc: the summary query lives in a device array of the library's own ----
// One copy of the array exists on every GPU the library runs on, at an address of that GPU's own; in host code the
// array's name is only a handle for hipGetSymbolAddress, never a pointer to pass on.
constexpr size_t STATIC_SCRATCH_BYTES = 256 * 1024;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up once per device).
lca_status static_scratch(void **out)
{
    int dev = -1;
    LCA_TRY(hip_status(hipGetDevice(&dev), "hipGetDevice"));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(LCA_ERR_UNSUPPORTED, "device ordinal %d is beyond the %d this library keeps scratch addresses for", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        LCA_TRY(hip_status(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"));
        if (p == nullptr) return fail(LCA_ERR_HIP, "hipGetSymbolAddress(scratch) returned a NULL address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LCA_OK;
}

}  // namespace

extern "C" {

lca_status lca_probe_hbm_read(const void *buf, size_t bytes, uint32_t *wg_sums, void *stream)
{
    LCA_TRY(check_ptr(buf, "buf"));
    if (wg_sums == nullptr) return fail(LCA_ERR_INVALID_ARG, "wg_sums is NULL");
    if (bytes == 0 || bytes % 16 != 0) return fail(LCA_ERR_INVALID_ARG, "bytes (%zu) must be a positive multiple of 16", bytes);
    return LCA_LAUNCH(lca::launch_probe_hbm_read(buf, bytes, wg_sums, static_cast<hipStream_t>(stream)), "lca_probe_hbm_read");
}

lca_status lca_probe_mfma_bf16(int32_t iters, int32_t pattern, float *out, int32_t *wavefronts, void *stream)
{
    if (out == nullptr || wavefronts == nullptr) return fail(LCA_ERR_INVALID_ARG, "output pointer is NULL");
    if (iters < 1 || iters > 65536) return fail(LCA_ERR_INVALID_ARG, "iters (%d) must be in [1, 65536]", iters);
    if (pattern != 0 && pattern != 1) return fail(LCA_ERR_INVALID_ARG, "pattern (%d) must be 0 or 1", pattern);
    int waves = 0;
    (void)hipGetLastError();       // (see LCA_LAUNCH)
    const hipError_t e = lca::launch_probe_mfma_bf16(iters, pattern, out, &waves, static_cast<hipStream_t>(stream));
    *wavefronts = waves;
    return hip_status(e, "lca_probe_mfma_bf16");
}

const char *lca_last_error(void) { return g_err; }

lca_status lca_workspace_size(const lca_desc *desc, size_t *bytes)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (bytes == nullptr) return fail(LCA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = workspace_bytes(d);
    return LCA_OK;
}

lca_status lca_cache_bytes(const lca_desc *desc, size_t *dense_bytes, size_t *condensed_bytes)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (dense_bytes == nullptr || condensed_bytes == nullptr) return fail(LCA_ERR_INVALID_ARG, "output pointer is NULL");
    const size_t row = (size_t)(d.d_pool + d.d_sel) * d.elt;
    *dense_bytes = (size_t)d.B * d.L * d.P * row;
    *condensed_bytes = (size_t)d.B * ((size_t)d.S * d.m + (size_t)d.P * d.k) * row;
    return LCA_OK;
}

lca_status lca_condensed_rows(const lca_desc *desc, int32_t *m, int32_t *k)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (m == nullptr || k == nullptr) return fail(LCA_ERR_INVALID_ARG, "output pointer is NULL");
    *m = d.m;
    *k = d.k;
    return LCA_OK;
}

lca_status lca_condense(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL, void *pool_rep, void *sel_rep,
                        int32_t *anchor_idx, float *alpha_dbg, void *workspace, size_t workspace_bytes_, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (d.n_q > d.L) return fail(LCA_ERR_INVALID_ARG, "n_q (%d) must be in [1, L]", d.n_q);
    LCA_TRY(check_ptr(Q, "Q"));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    if (d.m > 0 && anchor_idx == nullptr) return fail(LCA_ERR_INVALID_ARG, "anchor_idx is NULL");
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::CondenseArgs a;
    a.d = d; a.Q = Q; a.POOL = POOL; a.SEL = SEL; a.pool_rep = pool_rep; a.sel_rep = sel_rep;
    a.anchor = anchor_idx; a.alpha_dbg = alpha_dbg; a.qbar = static_cast<float *>(workspace);
    return LCA_LAUNCH(lca::launch_condense(a, static_cast<hipStream_t>(stream)), "lca_condense");
}

lca_status lca_condense_noalloc(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL, void *pool_rep, void *sel_rep,
                                int32_t *anchor_idx, float *alpha_dbg, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (d.n_q > d.L) return fail(LCA_ERR_INVALID_ARG, "n_q (%d) must be in [1, L]", d.n_q);
    LCA_TRY(check_ptr(Q, "Q"));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    if (d.m > 0 && anchor_idx == nullptr) return fail(LCA_ERR_INVALID_ARG, "anchor_idx is NULL");
    if (qbar_bytes(d) > STATIC_SCRATCH_BYTES)
        return fail(LCA_ERR_WORKSPACE, "lca_condense_noalloc: the summary queries of this descriptor need %zu bytes (B * S * d_qk floats), the "
                                       "built-in scratch holds %zu; use lca_condense with a workspace of the caller's", qbar_bytes(d), STATIC_SCRATCH_BYTES);
    void *qbar = nullptr;
    LCA_TRY(static_scratch(&qbar));
    lca::CondenseArgs a;
    a.d = d; a.Q = Q; a.POOL = POOL; a.SEL = SEL; a.pool_rep = pool_rep; a.sel_rep = sel_rep;
    a.anchor = anchor_idx; a.alpha_dbg = alpha_dbg; a.qbar = static_cast<float *>(qbar);
    // (nothing in the scratch has to start at zero: the first kernel writes every summary query before the second reads it)
    return LCA_LAUNCH(lca::launch_condense(a, static_cast<hipStream_t>(stream)), "lca_condense_noalloc");
}

lca_status lca_prefill_attn(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL, const void *pool_rep,
                            const void *sel_rep, void *O, float *lse, void *workspace, size_t workspace_bytes_, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    LCA_TRY(check_ptr(Q, "Q"));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    LCA_TRY(check_ptr(O, "O"));
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::AttnArgs a;
    a.d = d; a.Q = Q; a.POOL = POOL; a.SEL = SEL; a.pool_rep = pool_rep; a.sel_rep = sel_rep; a.O = O; a.lse = lse; a.dense = 0;
    return run_attn(a, static_cast<hipStream_t>(stream), "lca_prefill_attn");
}

lca_status lca_prefill_attn_up(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL, const void *pool_rep,
                               const void *sel_rep, const void *W_up, void *O_up, float *lse, void *workspace, size_t workspace_bytes_,
                               void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (!lca::attn_mla_supported(d))
        return fail(LCA_ERR_UNSUPPORTED, "lca_prefill_attn_up is built for the MLA widths (512 + 64) in a 16-bit type, up-projection to 128 per head");
    LCA_TRY(check_ptr(Q, "Q"));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    LCA_TRY(check_ptr(W_up, "W_up"));
    LCA_TRY(check_ptr(O_up, "O_up"));
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::AttnArgs a;
    a.d = d; a.Q = Q; a.POOL = POOL; a.SEL = SEL; a.pool_rep = pool_rep; a.sel_rep = sel_rep; a.O = O_up; a.lse = lse; a.dense = 0;
    a.W_up = W_up;
    a.up_scratch = workspace;
    return LCA_LAUNCH(lca::launch_attn_mla(a, static_cast<hipStream_t>(stream)), "lca_prefill_attn_up");
}

lca_status dense_mla_attn(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL, void *O, float *lse,
                          void *workspace, size_t workspace_bytes_, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    LCA_TRY(check_ptr(Q, "Q"));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(O, "O"));
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    d.m = 0;            // no representatives: every row attends all tokens i <= t
    d.k = d.L;
    lca::AttnArgs a;
    a.d = d; a.Q = Q; a.POOL = POOL; a.SEL = SEL; a.pool_rep = nullptr; a.sel_rep = nullptr; a.O = O; a.lse = lse; a.dense = 1;
    return run_attn(a, static_cast<hipStream_t>(stream), "dense_mla_attn");
}

static lca_status check_layout(const lca::Dims &d, const lca_cache_layout *layout, int k_needed)
{
    if (layout == nullptr) return fail(LCA_ERR_INVALID_ARG, "layout is NULL");
    if (layout->m_cap < d.m) return fail(LCA_ERR_INVALID_ARG, "m_cap (%d) is below the number of representatives (%d)", layout->m_cap, d.m);
    if (layout->k_cap < k_needed) return fail(LCA_ERR_INVALID_ARG, "k_cap (%d) is below the number of raw tail tokens (%d)", layout->k_cap, k_needed);
    if (layout->k_start < 0 || layout->k_start >= layout->k_cap) return fail(LCA_ERR_INVALID_ARG, "k_start (%d) is outside [0, k_cap)", layout->k_start);
    return LCA_OK;
}

static lca_status decode_common(const lca_desc *desc, const lca_cache_layout *layout, const void *q, const void *pool_rep, const void *sel_rep,
                                const void *pool_tail, const void *sel_tail, void *O, void *workspace, size_t workspace_bytes_, void *stream,
                                const char *what)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (!lca::decode_supported(d))
        return fail(LCA_ERR_UNSUPPORTED, "%s has no kernel for this mode / dtype / widths / heads-per-set combination", what);
    if (layout != nullptr) LCA_TRY(check_layout(d, layout, d.k));
    LCA_TRY(check_ptr(q, "q"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    LCA_TRY(check_ptr(pool_tail, "pool_tail"));
    LCA_TRY(check_ptr(sel_tail, "sel_tail"));
    LCA_TRY(check_ptr(O, "O"));
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::DecodeArgs a;
    a.d = d; a.q = q; a.pool_rep = pool_rep; a.sel_rep = sel_rep; a.pool_tail = pool_tail; a.sel_tail = sel_tail; a.O = O;
    a.part = static_cast<float *>(workspace);
    a.splits = lca::decode_splits(d);
    a.m_cap = layout ? layout->m_cap : d.m;
    a.k_cap = layout ? layout->k_cap : d.k;
    a.k_start = layout ? layout->k_start : 0;
    return LCA_LAUNCH(lca::launch_decode(a, static_cast<hipStream_t>(stream)), what);
}

lca_status lca_decode_attn(const lca_desc *desc, const void *q, const void *pool_rep, const void *sel_rep, const void *pool_tail,
                           const void *sel_tail, void *O, void *workspace, size_t workspace_bytes_, void *stream)
{
    return decode_common(desc, nullptr, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, workspace_bytes_, stream, "lca_decode_attn");
}

lca_status lca_decode_attn_cached(const lca_desc *desc, const lca_cache_layout *layout, const void *q, const void *pool_rep, const void *sel_rep,
                                  const void *pool_tail, const void *sel_tail, void *O, void *workspace, size_t workspace_bytes_, void *stream)
{
    if (layout == nullptr) return fail(LCA_ERR_INVALID_ARG, "layout is NULL");
    return decode_common(desc, layout, q, pool_rep, sel_rep, pool_tail, sel_tail, O, workspace, workspace_bytes_, stream, "lca_decode_attn_cached");
}

lca_status lca_cache_update(const lca_desc *desc, const lca_cache_layout *layout, const void *q_recent, const void *pool_tail,
                            const void *sel_tail, void *pool_rep, void *sel_rep, int32_t *anchor_idx, void *workspace, size_t workspace_bytes_,
                            void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (d.L < d.w + d.g || (d.L - d.w) % d.g != 0)
        return fail(LCA_ERR_INVALID_ARG, "no update is due at L = %d (w = %d, g = %d): needs L >= w + g and (L - w) mod g == 0", d.L, d.w, d.g);
    if (d.n_q > d.L) return fail(LCA_ERR_INVALID_ARG, "n_q (%d) must be in [1, L]", d.n_q);
    if (d.pool_reduce != LCA_REDUCE_WEIGHTED || d.sel_reduce != LCA_REDUCE_MAXSEL)
        return fail(LCA_ERR_UNSUPPORTED, "lca_cache_update is built for the method's own strategies only (weighted pooling, max selection)");
    LCA_TRY(check_layout(d, layout, d.w + d.g));
    LCA_TRY(check_ptr(q_recent, "q_recent"));
    LCA_TRY(check_ptr(pool_tail, "pool_tail"));
    LCA_TRY(check_ptr(sel_tail, "sel_tail"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep"));
    LCA_TRY(check_ptr(sel_rep, "sel_rep"));
    if (anchor_idx != nullptr && (reinterpret_cast<uintptr_t>(anchor_idx) & 3)) return fail(LCA_ERR_INVALID_ARG, "anchor_idx is not 4-byte aligned");
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::UpdateArgs a;
    a.qbar = static_cast<float *>(workspace);
    a.d = d; a.q_recent = q_recent; a.pool_tail = pool_tail; a.sel_tail = sel_tail; a.pool_rep = pool_rep; a.sel_rep = sel_rep;
    a.anchor = anchor_idx; a.m_cap = layout->m_cap; a.k_cap = layout->k_cap; a.k_start = layout->k_start;
    return LCA_LAUNCH(lca::launch_cache_update(a, static_cast<hipStream_t>(stream)), "lca_cache_update");
}

lca_status lca_quantize_cache(const lca_desc *desc, const lca_cache_layout *layout, int32_t first_row, const void *pool_rep, const void *sel_rep,
                              uint8_t *pool_q8, uint8_t *sel_q8, float *scales, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (d.dtype == LCA_F32) return fail(LCA_ERR_UNSUPPORTED, "lca_quantize_cache reads a 16-bit cache");
    if (layout != nullptr) LCA_TRY(check_layout(d, layout, d.k));
    if (first_row < 0 || first_row > d.m) return fail(LCA_ERR_INVALID_ARG, "first_row (%d) must be in [0, m = %d]", first_row, d.m);
    if (first_row == d.m) return LCA_OK;
    LCA_TRY(check_ptr(pool_rep, "pool_rep"));
    LCA_TRY(check_ptr(sel_rep, "sel_rep"));
    LCA_TRY(check_ptr(pool_q8, "pool_q8"));
    LCA_TRY(check_ptr(sel_q8, "sel_q8"));
    if (scales == nullptr || (reinterpret_cast<uintptr_t>(scales) & 7)) return fail(LCA_ERR_INVALID_ARG, "scales is NULL or not 8-byte aligned");
    lca::QuantArgs a;
    a.d = d; a.pool_rep = pool_rep; a.sel_rep = sel_rep; a.pool_q8 = pool_q8; a.sel_q8 = sel_q8; a.scales = scales;
    a.m_cap = layout ? layout->m_cap : d.m;
    a.first_row = first_row;
    return LCA_LAUNCH(lca::launch_quantize_cache(a, static_cast<hipStream_t>(stream)), "lca_quantize_cache");
}

lca_status lca_decode_attn_q8(const lca_desc *desc, const lca_cache_layout *layout, const void *q, const uint8_t *pool_q8, const uint8_t *sel_q8,
                              const float *scales, const void *pool_tail, const void *sel_tail, void *O, void *workspace, size_t workspace_bytes_,
                              void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    if (!lca::decode_mla_supported(d) && !lca::decode_gqa_mfma_supported(d))
        return fail(LCA_ERR_UNSUPPORTED,
                    "lca_decode_attn_q8 is built for the MLA widths (512 + 64) and the GQA widths (128 / 128) in a 16-bit type with at most 16 heads per set");
    if (layout != nullptr) LCA_TRY(check_layout(d, layout, d.k));
    LCA_TRY(check_ptr(q, "q"));
    LCA_TRY(check_ptr(pool_q8, "pool_q8", d.m > 0));
    LCA_TRY(check_ptr(sel_q8, "sel_q8", d.m > 0));
    if (d.m > 0 && (scales == nullptr || (reinterpret_cast<uintptr_t>(scales) & 7))) return fail(LCA_ERR_INVALID_ARG, "scales is NULL or not 8-byte aligned");
    LCA_TRY(check_ptr(pool_tail, "pool_tail"));
    LCA_TRY(check_ptr(sel_tail, "sel_tail"));
    LCA_TRY(check_ptr(O, "O"));
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::DecodeArgs a;
    a.d = d; a.q = q; a.pool_rep = nullptr; a.sel_rep = nullptr; a.pool_tail = pool_tail; a.sel_tail = sel_tail; a.O = O;
    a.pool_q8 = pool_q8; a.sel_q8 = sel_q8; a.scales = scales;
    a.part = static_cast<float *>(workspace);
    a.splits = lca::decode_splits(d);
    a.m_cap = layout ? layout->m_cap : d.m;
    a.k_cap = layout ? layout->k_cap : d.k;
    a.k_start = layout ? layout->k_start : 0;
    // (with m = 0 there are no representatives: the kernel for the 16-bit cache reads the tail alone)
    if (d.m == 0) { a.pool_q8 = nullptr; a.sel_q8 = nullptr; a.scales = nullptr; }
    return LCA_LAUNCH(lca::launch_decode(a, static_cast<hipStream_t>(stream)), "lca_decode_attn_q8");
}

lca_status lca_deviation_stats(const lca_desc *desc, const void *POOL, const void *SEL, const void *pool_rep, const void *sel_rep, float *stats,
                               void *workspace, size_t workspace_bytes_, void *stream)
{
    lca::Dims d;
    LCA_TRY(make_dims(desc, d));
    LCA_TRY(check_ptr(POOL, "POOL"));
    LCA_TRY(check_ptr(SEL, "SEL"));
    LCA_TRY(check_ptr(pool_rep, "pool_rep", d.m > 0));
    LCA_TRY(check_ptr(sel_rep, "sel_rep", d.m > 0));
    if (stats == nullptr || (reinterpret_cast<uintptr_t>(stats) & 3)) return fail(LCA_ERR_INVALID_ARG, "stats is NULL or not 4-byte aligned");
    LCA_TRY(check_ws(d, workspace, workspace_bytes_));
    lca::DeviationArgs a;
    a.d = d; a.POOL = POOL; a.SEL = SEL; a.pool_rep = pool_rep; a.sel_rep = sel_rep; a.stats = stats;
    a.partial = static_cast<float *>(workspace);
    return LCA_LAUNCH(lca::launch_deviation_stats(a, static_cast<hipStream_t>(stream)), "lca_deviation_stats");
}

}  // extern "C"
