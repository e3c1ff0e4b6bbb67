/*
 * liblca — Latent-Condensed Attention (LCA) hot path for AMD MI355X (gfx950), C ABI.
 *
 * Notation follows the paper: L tokens, group size g, local window w, m = floor((L - w) / g)
 * groups (0 when L <= w), k = L - m*g raw tokens (section 4.2; Algorithm 1).  Indices are 0-based:
 * group j covers tokens [j*g, (j+1)*g).
 *
 * Modes
 *   LCA_MODE_MLA  POOL = C^KV [B, L, d_pool], SEL = K^R [B, L, d_sel], shared by all heads.  Absorbed
 *                 form (section 3, Eq. 2-5 with W^UK, W^UV folded away): key_i = [c_i ; k^R_i],
 *                 d_qk = d_pool + d_sel, value_i = c_i, d_v = d_pool.
 *   LCA_MODE_GQA  POOL = V, SEL = K, both [B, L, S, d] with one condensed set per KV head
 *                 (section 5.4: max-selection on keys, weighted pooling on values); d_qk = d_sel,
 *                 d_v = d_pool.
 * Condensed sets: S per sequence, query head h uses set h / (H / S).  S = 1 (MLA) or S = KV heads
 * (GQA) reproduces the cache sizes the paper reports; S = H condenses per query head.
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers, row-major, last dimension contiguous, 16-byte
 *     aligned; `desc` and size outputs are HOST pointers.  Element type is desc->dtype for Q, POOL,
 *     SEL, the representatives and O; anchor indices are int32; lse and alpha_dbg are float.
 *   - The caller owns every buffer, including the workspace (size from lca_workspace_size).  The
 *     library allocates nothing, keeps no state between calls and never synchronises: work is
 *     enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream) and outputs are
 *     valid once the caller has synchronised that stream.
 *   - Every call returns an lca_status.  On any status other than LCA_OK nothing was launched and no
 *     output was touched, except LCA_ERR_HIP, which reports a launch failure from the HIP runtime.
 *     lca_last_error() gives a thread-local message for the last non-OK status.
 *   - Invalid: NULL required pointer; B, L, H, S, g <= 0; w < 0; H % S != 0; n_q < 0, and n_q > L in
 *     the calls that read the summary queries (lca_condense, lca_cache_update); a dtype or
 *     mode outside the enums; d_pool / d_sel not multiples of 8 (bf16, f16) or 4 (f32) or above 1024;
 *     g > 64; a reduce strategy outside the enum; workspace too small (LCA_ERR_WORKSPACE).  m = 0 (L < w + g) is valid: lca_condense
 *     writes nothing and lca_prefill_attn equals dense attention (section 4.3, fallback remark).
 */
#ifndef LCA_H
#define LCA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LCA_OK = 0,
    LCA_ERR_INVALID_ARG = 1,
    LCA_ERR_UNSUPPORTED = 2,
    LCA_ERR_WORKSPACE = 3,
    LCA_ERR_HIP = 4
} lca_status;

typedef enum { LCA_MODE_MLA = 0, LCA_MODE_GQA = 1 } lca_mode;
/* Element type of Q, POOL, SEL, the representatives and O.  The two 16-bit types are the ones the paper's
 * implementation is written for (limitations section); products are accumulated in fp32 for all three. */
typedef enum { LCA_BF16 = 0, LCA_F32 = 1, LCA_F16 = 2 } lca_dtype;

/*
 * How the g vectors of a group become the representative's component (the ablation of section 5.4,
 * Table 5; appendix "Comparison with Alternative Pooling Strategies").  LCA_REDUCE_DEFAULT is the
 * method: weighted pooling for the pooled component (Eq. 7), max selection for the selected one (Eq. 8).
 *   WEIGHTED  sum_i alpha_i x_i with the group softmax alpha of Eq. 6
 *   MEAN      (1/g) sum_i x_i
 *   MAXSEL    x of the token with the largest importance score (lowest index on ties), copied
 *   MAXPOOL   the x of largest Euclidean norm in the group (lowest index on ties), copied — the appendix
 *             describes max pooling as keeping "the vector with the highest norm"
 * Only lca_condense reads these fields; anchor_idx always reports the arg-max score token.
 */
typedef enum {
    LCA_REDUCE_DEFAULT = 0, LCA_REDUCE_WEIGHTED = 1, LCA_REDUCE_MEAN = 2, LCA_REDUCE_MAXSEL = 3, LCA_REDUCE_MAXPOOL = 4
} lca_reduce;

typedef struct {
    int32_t B, L, H, S;     /* batch, tokens, query heads, condensed sets (H % S == 0)            */
    int32_t d_pool, d_sel;  /* widths of the pooled and of the selected component                  */
    int32_t g, w, n_q;      /* group size, local window, number of summary queries (0 means g)     */
    int32_t mode, dtype;    /* lca_mode, lca_dtype                                                 */
    float scale;            /* multiplies q.k in the importance score and in the attention logits  */
    float rep_logit_bias;   /* added to representatives' logits: 0 = Algorithm 1; ln(g) = each
                               representative counted g times, the normaliser used in appendix A.2 */
    int32_t pool_reduce;    /* lca_reduce for the pooled component   (0 = weighted pooling)        */
    int32_t sel_reduce;     /* lca_reduce for the selected component (0 = max selection)           */
} lca_desc;

/* Bytes of workspace that any call below needs for this descriptor (host only, launches nothing). */
lca_status lca_workspace_size(const lca_desc *desc, size_t *bytes);

/*
 * The partition of section 4.2 (Algorithm 1: groups, then local window plus remainder) for this descriptor:
 * m = floor((L - w) / g) groups (0 when L <= w) and k = L - m*g raw tokens, so that m*g + k = L.  These are the
 * row counts of every representative buffer ([B,S,m,.]) and raw tail ([B,P,k,.]) in the calls below.  Host only.
 */
lca_status lca_condensed_rows(const lca_desc *desc, int32_t *m, int32_t *k);

/*
 * KV-cache footprint of one layer (section 4.3, decoding paragraph; appendix B): dense = one
 * (pool, sel) row per token and KV head; condensed = S*m representatives plus k raw tail rows per
 * KV head.  Host only.
 */
lca_status lca_cache_bytes(const lca_desc *desc, size_t *dense_bytes, size_t *condensed_bytes);

/*
 * Latent-space condensation (section 4.2; Algorithm 1, first step and loop over groups).
 *   summary query  qbar[b,s,:] = mean of Q[b, L-n_q .. L-1, heads of set s, :]
 *   score          s_i = scale * <qbar, key_i>,  alpha = softmax of s inside each group   (Eq. 6)
 *   pool_rep[b,s,j,:] = sum_i alpha_i * POOL_i                                             (Eq. 7)
 *   anchor_idx[b,s,j] = lowest token index attaining max s_i, sel_rep[b,s,j,:] = SEL row of it (Eq. 8)
 * In:  Q [B,L,H,d_qk], POOL, SEL (layouts above).
 * Out: pool_rep [B,S,m,d_pool], sel_rep [B,S,m,d_sel] (dtype of the inputs, pooled values rounded
 *      to nearest-even once on store), anchor_idx [B,S,m] (absolute token index),
 *      alpha_dbg [B,S,m*g] float, may be NULL.  With m = 0 nothing is written.
 */
lca_status lca_condense(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL,
                        void *pool_rep, void *sel_rep, int32_t *anchor_idx, float *alpha_dbg,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * lca_condense for callers that can neither allocate device memory nor hand over a workspace: code under HIP graph
 * capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc.  Same inputs, outputs and results
 * as lca_condense; the summary queries (B * S * d_qk floats, the only scratch memory that call uses) live in a device
 * array built into the library instead of the caller's workspace.  The call allocates nothing and frees nothing.
 *   - Limit: B * S * d_qk * 4 bytes (rounded up to 256) must not exceed 256 KiB, e.g. B * S <= 113 at d_qk = 576;
 *     beyond it the call returns LCA_ERR_WORKSPACE and launches nothing.
 *   - Every GPU the library runs on holds its own copy of the array for the life of the process; its address on the
 *     current device is looked up on the first call made with that device current (make that call outside a capture).
 *   - All calls on one GPU share the array, which keeps the previous call's contents; nothing in it has to start at
 *     zero.  Two calls whose kernels overlap on one GPU (different streams, no ordering between them) race on it:
 *     order them, or use lca_condense with separate workspaces.
 */
lca_status lca_condense_noalloc(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL,
                                void *pool_rep, void *sel_rep, int32_t *anchor_idx, float *alpha_dbg, void *stream);

/*
 * Prefill attention over the condensed context (section 4.3, Eq. 10; Algorithm 1, last steps;
 * appendix A.2 notation for a query at position t).  Row t of head h (set s) attends
 *   representatives j < m_t,  m_t = max(0, floor((t + 1 - w) / g)),  and raw tokens m_t*g <= i <= t,
 * with one softmax over both; logits scale*<q, key> (+ rep_logit_bias on representatives); the
 * output is the probability-weighted sum of pool_rep rows and raw POOL rows (latent space for MLA).
 * In:  Q [B,L,H,d_qk], POOL, SEL, pool_rep, sel_rep (as written by lca_condense).
 * Out: O [B,L,H,d_pool]; lse [B,L,H] float (natural-log normaliser of the scaled logits), may be NULL.
 */
lca_status lca_prefill_attn(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL,
                            const void *pool_rep, const void *sel_rep, void *O, float *lse,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * lca_prefill_attn with the head's value up-projection applied before the output is written (section 3, Eq. 5:
 * o_t = (sum_i p_i c_i) W^UV -- the matrix the absorbed form leaves to the output side; Algorithm 1 keeps it
 * outside the attention).  The kernel multiplies while the latent output of its rows is still in registers, so the
 * output is a quarter of the size and the separate projection pass over O is saved.  The latent output is rounded
 * once to desc->dtype before the product, as it would be if it were stored and projected afterwards.
 * In:  as lca_prefill_attn, plus W_up [H, 128, d_pool]: row u of head h holds W^UV_h[:, u] (output dimension major,
 *      the layout of a linear layer's weight).
 * Out: O_up [B,L,H,128]; lse as there.
 * Built for the MLA widths (d_pool = 512, d_sel = 64) in bf16 or fp16; other shapes return LCA_ERR_UNSUPPORTED.
 */
lca_status lca_prefill_attn_up(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL,
                               const void *pool_rep, const void *sel_rep, const void *W_up, void *O_up, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Dense causal attention, the in-run baseline (section 3, Eq. 5; absorbed form for MLA): row t
 * attends every token i <= t.  desc->g, w, n_q and rep_logit_bias are ignored.  Same layouts as
 * lca_prefill_attn without the representatives.
 */
lca_status dense_mla_attn(const lca_desc *desc, const void *Q, const void *POOL, const void *SEL,
                          void *O, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step over a condensed cache (section 4.3, decoding paragraph).  desc->L is the number
 * of tokens so far INCLUDING the new one, whose key/value the caller has appended to the raw tail;
 * the library derives m = floor((L - w) / g) and the tail length k = L - m*g.  The new token's
 * query attends the m representatives and the k tail rows.
 * In:  q [B,H,d_qk]; pool_rep [B,S,m,d_pool], sel_rep [B,S,m,d_sel];
 *      pool_tail [B,P,k,d_pool], sel_tail [B,P,k,d_sel] with P = 1 (MLA) or S (GQA).
 * Out: O [B,H,d_pool].
 * Built for: the MLA widths (512 + 64) and the GQA widths (128 / 128) in bf16 or fp16 with at most 16 query
 * heads per condensed set (matrix-core kernels); MLA 512 + 64 with one set per head or 16 heads per set, and
 * fp32 MLA 128 + 32 with 1 or 4 heads per set (general kernel).  Other shapes return LCA_ERR_UNSUPPORTED.
 */
lca_status lca_decode_attn(const lca_desc *desc, const void *q, const void *pool_rep, const void *sel_rep,
                           const void *pool_tail, const void *sel_tail, void *O,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * A decoding batch's cache as it grows (section 4.3, "Decoding and Online Cache Update"): the buffers
 * are allocated once with room for more rows than are in use, and the raw tail is a ring.
 *   pool_rep [B,S,m_cap,d_pool], sel_rep [B,S,m_cap,d_sel], anchor_idx [B,S,m_cap]: rows [0, m) in use;
 *   pool_tail [B,P,k_cap,d_pool], sel_tail [B,P,k_cap,d_sel]: raw token number i of the tail (0 = oldest)
 *   sits in ring row (k_start + i) mod k_cap.
 * Writing a new token's rows into the ring (row (k_start + k) mod k_cap before the step) is the
 * caller's business, as in lca_decode_attn.
 */
typedef struct {
    int32_t m_cap;      /* representative rows allocated per (sequence, set);  m <= m_cap            */
    int32_t k_cap;      /* tail rows allocated per (sequence, KV head);        k <= k_cap            */
    int32_t k_start;    /* ring row of the oldest raw token, 0 <= k_start < k_cap                    */
} lca_cache_layout;

/*
 * lca_decode_attn over a cache with the layout above; m and k follow from desc->L as there.
 * Invalid in addition: m > m_cap, k > k_cap, k_start outside [0, k_cap).
 */
lca_status lca_decode_attn_cached(const lca_desc *desc, const lca_cache_layout *layout, const void *q,
                                  const void *pool_rep, const void *sel_rep, const void *pool_tail,
                                  const void *sel_tail, void *O, void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * Online cache update (section 4.3, same paragraph): once g new tokens have arrived, the g oldest
 * raw tokens of the tail are condensed into one more representative, scored with the mean query of
 * the last n_q (default g) tokens as in Eq. 6 and reduced by Eq. 7 and Eq. 8.
 * desc->L = tokens so far INCLUDING the newest, already in the ring; the call is due exactly when
 * L >= w + g and (L - w) mod g == 0.  With m = (L - w) / g, the ring holds the w + g tokens
 * [(m-1)*g, L) before the call; the call writes row m-1 of pool_rep, sel_rep and anchor_idx (the
 * anchor as an absolute token index) and touches nothing else.  Afterwards the cache is the one
 * lca_decode_attn_cached expects for this L with k_start advanced by g (mod k_cap): m
 * representatives and the w newest raw tokens; the g condensed ring rows are free for new tokens.
 * In:  q_recent [B,n_q,H,d_qk], oldest first; pool_tail, sel_tail (the ring, read only).
 * Out: row m-1 of pool_rep [B,S,m_cap,d_pool], sel_rep [B,S,m_cap,d_sel], anchor_idx [B,S,m_cap] (may be NULL).
 * Invalid in addition: L < w + g or (L - w) mod g != 0; m > m_cap; w + g > k_cap; k_start outside [0, k_cap).
 * Workspace: lca_workspace_size(desc) bytes (the summary query lives there).
 */
lca_status lca_cache_update(const lca_desc *desc, const lca_cache_layout *layout, const void *q_recent,
                            const void *pool_tail, const void *sel_tail, void *pool_rep, void *sel_rep,
                            int32_t *anchor_idx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Per-token deviations between the original keys / values and the representative standing for them:
 * the delta_k, delta_v of the error bound (section 4.4, Theorem 1), measured as in the appendix on
 * empirical per-token deviations (Tables 9-10).  For every condensed token i of group j (i < m*g):
 *     dk_i = || key_i - key^rep_j ||_2,   dv_i = || value_i - value^rep_j ||_2,
 * key = [pool ; sel] (MLA, the absorbed space attention works in) or sel (GQA), value = pool.
 * In:  POOL, SEL, pool_rep, sel_rep as for lca_prefill_attn.
 * Out: stats [B,S,6] float = mean dk, mean dk/||key_i||, max dk, mean dv, mean dv/||value_i||, max dv over
 *      those tokens (a ratio with a zero denominator counts as 0; all zeros when m = 0).
 * Deterministic: per-group sums go through the workspace and are added in a fixed order.
 */
lca_status lca_deviation_stats(const lca_desc *desc, const void *POOL, const void *SEL, const void *pool_rep,
                               const void *sel_rep, float *stats, void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * 8-bit copy of the representatives, for decoding over a cache half the size (the paper's limitations section
 * names lower precisions as unexplored: the format is this library's).  Codes are OCP FP8 E4M3 bytes; every
 * representative row has one power-of-two scale per component, chosen so that the row's largest magnitude
 * lands in (224, 448] (1 for an all-zero row); a value x is stored as the code nearest to x / scale (ties to
 * even, the sign of x kept) and stands for decode(code) * scale.  The raw tail stays in the 16-bit type.
 * desc->L, the layout (may be NULL: m_cap = m) and the row counts are those of lca_decode_attn_cached; only
 * rows [first_row, m) of every (sequence, set) are read and written (0 after a prefill; m - 1 after an
 * lca_cache_update, which adds row m - 1).  desc->dtype must be a 16-bit type.  Invalid in addition:
 * first_row outside [0, m].
 * In:  pool_rep [B,S,m_cap,d_pool], sel_rep [B,S,m_cap,d_sel].
 * Out: pool_q8 [B,S,m_cap,d_pool], sel_q8 [B,S,m_cap,d_sel] bytes (8-byte aligned rows: d_pool, d_sel are multiples
 *      of 8), scales [B,S,m_cap,2] float (pooled, selected).
 */
lca_status lca_quantize_cache(const lca_desc *desc, const lca_cache_layout *layout, int32_t first_row, const void *pool_rep,
                              const void *sel_rep, uint8_t *pool_q8, uint8_t *sel_q8, float *scales, void *stream);

/*
 * lca_decode_attn_cached over the 8-bit representatives lca_quantize_cache wrote (layout may be NULL: m_cap = m,
 * k_cap = k, k_start = 0); the raw tail is read in desc->dtype as there.  Each stored value enters the products as
 * decode(code) * scale, which is exact in either 16-bit type; everything else is the decode step of section 4.3.
 * Built for the MLA widths (d_pool = 512, d_sel = 64) and the GQA widths (128 / 128), a 16-bit dtype, at most 16
 * heads per set; other shapes return LCA_ERR_UNSUPPORTED.
 */
lca_status lca_decode_attn_q8(const lca_desc *desc, const lca_cache_layout *layout, const void *q, const uint8_t *pool_q8,
                              const uint8_t *sel_q8, const float *scales, const void *pool_tail, const void *sel_tail,
                              void *O, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aids, not steps of the method: what the device sustains at the two operations the roofline fractions
 * of the kernels above are read against (the measured-ceiling lines asked for beside the published peaks).  Time
 * them from outside, with events on the stream they are given.
 *
 * lca_probe_hbm_read streams `bytes` bytes (a positive multiple of 16, buf 16-byte aligned, device memory) once, with
 * the launch shape that read fastest on gfx950, and leaves in wg_sums (device, LCA_PROBE_WORDS words) per-workgroup
 * sums of the 32-bit words read: their total modulo 2^32 is the sum of all words of the buffer; unused entries are 0.
 *
 * lca_probe_mfma_bf16 runs, on every SIMD of the device, iters (1 .. 65536) rounds of four independent
 * 32x32x16 bf16 matrix-core products with fp32 accumulation: chain c (0..3) accumulates D_c += A_c B_c, A_c 32 x 16,
 * B_c 16 x 32, constant over the rounds.
 *   pattern 0: A_c[i][k] = (5 i + 3 c) mod 7 - 2, B_c[k][j] = (3 j + 5 c + 1) mod 7 - 2: every output element is the
 *              integer 16 iters A_c[i][0] B_c[0][j], exact in fp32.
 *   pattern 1: operands with all mantissa bits in use and mixed signs, as a real kernel's (the clock the device
 *              settles at under matrix-core load depends on how many operand bits toggle): element (x, k) of operand
 *              o (0 = A with x = i, 1 = B with x = j) of chain c has the bf16 bit pattern
 *              sign(h >> 31) | exponent 126 + ((h >> 8) & 1) | mantissa h & 127, where h = mix(((o 4 + c) 32 + x) 16 + k + 1),
 *              mix(x): x *= 2654435761; x ^= x >> 15; x *= 2246822519; x ^= x >> 13 (32-bit unsigned arithmetic).
 * *wavefronts (host) receives the number of wavefronts that ran; flops = wavefronts * iters * 4 * 32768.
 * out (device, LCA_PROBE_MFMA_FLOATS floats, the first wavefronts * 256 written): out[(64 v + l) * 4 + c] = the sum of
 * the 16 elements of D_c that lane l of wavefront v holds -- rows of column l mod 32, lanes l and l + 32 together the
 * whole column -- so out[(64 v + l) * 4 + c] + out[(64 v + l + 32) * 4 + c] = sum_i D_c[i][l] for l < 32.
 */
#define LCA_PROBE_WORDS 256
#define LCA_PROBE_MFMA_FLOATS (256 * 256 * 4)
lca_status lca_probe_hbm_read(const void *buf, size_t bytes, uint32_t *wg_sums, void *stream);
lca_status lca_probe_mfma_bf16(int32_t iters, int32_t pattern, float *out, int32_t *wavefronts, void *stream);

/* Message for the calling thread's last non-OK status; never NULL. */
const char *lca_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LCA_H */
