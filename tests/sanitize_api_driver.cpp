// Host-side validation of liblca under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).
// tests/test_sanitizers.py builds the whole library a second time with the sanitizers on its HOST code and links this
// program against it.  Every call below either is host-only (sizes, cache bytes, partition) or must be rejected by the
// argument checks before anything is launched, so the program needs no GPU; a sanitizer report ends it with a
// non-zero status.  Prints "checks N" at the end.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>

#include "lca.h"

static int n_checks = 0, n_bad = 0;
#define EXPECT(cond) do { ++n_checks; if (!(cond)) { ++n_bad; std::printf("FAILED line %d: %s  (last error: %s)\n", __LINE__, #cond, lca_last_error()); } } while (0)

static lca_desc mla(int B, int L, int H, int S, int g, int w)
{
    lca_desc d;
    std::memset(&d, 0, sizeof d);
    d.B = B; d.L = L; d.H = H; d.S = S; d.d_pool = 512; d.d_sel = 64; d.g = g; d.w = w; d.mode = LCA_MODE_MLA; d.dtype = LCA_BF16; d.scale = 1.f;
    return d;
}

int main()
{
    void *A = reinterpret_cast<void *>(0x10000);      // aligned, non-NULL, never dereferenced: validation must stop first
    size_t n = 0, a = 0, b = 0;
    int32_t m = 0, k = 0;
    lca_desc d = mla(1, 131072, 16, 1, 16, 1024);
    EXPECT(lca_workspace_size(&d, &n) == LCA_OK && n >= 576 * 4);
    EXPECT(lca_cache_bytes(&d, &a, &b) == LCA_OK && a == 150994944u && b == 10543104u);
    EXPECT(lca_condensed_rows(&d, &m, &k) == LCA_OK && m == 8128 && k == 1024);
    EXPECT(lca_workspace_size(nullptr, &n) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_workspace_size(&d, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_condensed_rows(&d, nullptr, &k) == LCA_ERR_INVALID_ARG);
    EXPECT(std::strlen(lca_last_error()) > 0);

    // descriptors at the edges of the integer range: sizes are computed in 64 bits or rejected, never overflowed
    const int big = std::numeric_limits<int32_t>::max();
    for (int which = 0; which < 8; ++which) {
        lca_desc e = mla(1, 4096, 16, 1, 16, 128);
        if (which == 0) e.B = big;
        if (which == 1) e.L = big;
        if (which == 2) { e.H = big; e.S = big; }
        if (which == 3) { e.B = 1 << 15; e.L = 1 << 15; e.H = 1 << 10; e.S = 1 << 10; }
        if (which == 4) e.w = big;
        if (which == 5) e.n_q = big;
        if (which == 6) { e.L = big; e.w = 0; e.g = 1; }
        if (which == 7) { e.B = 46340; e.L = 46340; e.H = 1; }
        const lca_status s1 = lca_workspace_size(&e, &n), s2 = lca_cache_bytes(&e, &a, &b), s3 = lca_condensed_rows(&e, &m, &k);
        EXPECT(s1 == LCA_OK || s1 == LCA_ERR_INVALID_ARG || s1 == LCA_ERR_UNSUPPORTED);
        EXPECT(s2 == s1 && s3 == s1);
        if (s3 == LCA_OK) EXPECT((int64_t)m * e.g + k == e.L && m >= 0 && k >= 0);
    }
    for (int field = 0; field < 12; ++field) {        // one invalid field at a time
        lca_desc e = mla(2, 1000, 8, 2, 16, 100);
        switch (field) {
        case 0: e.B = 0; break;
        case 1: e.L = -5; break;
        case 2: e.H = 7; break;
        case 3: e.g = 0; break;
        case 4: e.g = 65; break;
        case 5: e.w = -1; break;
        case 6: e.n_q = -1; break;
        case 7: e.mode = 2; break;
        case 8: e.dtype = 9; break;
        case 9: e.d_pool = 100; break;
        case 10: e.scale = std::numeric_limits<float>::quiet_NaN(); break;
        case 11: e.pool_reduce = 5; break;
        }
        EXPECT(lca_workspace_size(&e, &n) != LCA_OK);
        EXPECT(lca_condense(&e, A, A, A, A, A, static_cast<int32_t *>(A), nullptr, A, size_t(1) << 30, nullptr) != LCA_OK);
        EXPECT(lca_condense_noalloc(&e, A, A, A, A, A, static_cast<int32_t *>(A), nullptr, nullptr) != LCA_OK);
        EXPECT(lca_prefill_attn(&e, A, A, A, A, A, A, nullptr, A, size_t(1) << 30, nullptr) != LCA_OK);
    }

    // pointers: NULL, misaligned, workspace missing or short -- every entry point, before any launch
    d = mla(1, 8192, 16, 1, 16, 1024);
    EXPECT(lca_workspace_size(&d, &n) == LCA_OK);
    void *odd = reinterpret_cast<void *>(0x10002);
    int32_t *An = static_cast<int32_t *>(A);
    EXPECT(lca_condense(&d, nullptr, A, A, A, A, An, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_condense(&d, A, odd, A, A, A, An, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_condense(&d, A, A, A, A, A, nullptr, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_condense(&d, A, A, A, A, A, An, nullptr, nullptr, n, nullptr) == LCA_ERR_WORKSPACE);
    EXPECT(lca_condense(&d, A, A, A, A, A, An, nullptr, A, n - 1, nullptr) == LCA_ERR_WORKSPACE);
    EXPECT(lca_condense_noalloc(&d, A, A, nullptr, A, A, An, nullptr, nullptr) == LCA_ERR_INVALID_ARG);
    lca_desc wide = mla(8, 64, 16, 16, 4, 8);            // 8 * 16 * 576 floats: beyond the built-in scratch
    EXPECT(lca_condense_noalloc(&wide, A, A, A, A, A, An, nullptr, nullptr) == LCA_ERR_WORKSPACE);
    EXPECT(lca_prefill_attn(&d, A, A, A, A, A, nullptr, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_prefill_attn_up(&d, A, A, A, A, A, nullptr, A, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(dense_mla_attn(&d, A, nullptr, A, A, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_decode_attn(&d, nullptr, A, A, A, A, A, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    lca_cache_layout lay = {4, 80, 80};
    lca_desc upd = mla(1, 80, 16, 1, 16, 64);
    EXPECT(lca_cache_update(&upd, &lay, A, A, A, A, A, An, A, size_t(1) << 20, nullptr) == LCA_ERR_INVALID_ARG);   // k_start outside the ring
    lay.k_start = 0; lay.m_cap = 0;
    EXPECT(lca_cache_update(&upd, &lay, A, A, A, A, A, An, A, size_t(1) << 20, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_decode_attn_cached(&upd, nullptr, A, A, A, A, A, A, A, size_t(1) << 20, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_decode_attn_cached(&upd, &lay, A, A, A, A, A, A, A, size_t(1) << 20, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_quantize_cache(&upd, nullptr, 2, A, A, static_cast<uint8_t *>(A), static_cast<uint8_t *>(A), static_cast<float *>(A), nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_quantize_cache(&upd, nullptr, 1, A, A, static_cast<uint8_t *>(A), static_cast<uint8_t *>(A), static_cast<float *>(A), nullptr) == LCA_OK);   // nothing to do
    EXPECT(lca_decode_attn_q8(&upd, nullptr, nullptr, static_cast<uint8_t *>(A), static_cast<uint8_t *>(A), static_cast<float *>(A), A, A, A, A,
                              size_t(1) << 20, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_deviation_stats(&d, A, A, A, A, nullptr, A, n, nullptr) == LCA_ERR_INVALID_ARG);
    lca_desc odd_widths = mla(1, 100, 3, 1, 4, 4);
    odd_widths.d_pool = 64; odd_widths.d_sel = 64;
    EXPECT(lca_decode_attn(&odd_widths, A, A, A, A, A, A, A, size_t(1) << 20, nullptr) == LCA_ERR_UNSUPPORTED);
    EXPECT(lca_prefill_attn_up(&odd_widths, A, A, A, A, A, A, A, nullptr, A, size_t(1) << 20, nullptr) == LCA_ERR_UNSUPPORTED);
    // the measurement aids
    int32_t waves = -7;
    EXPECT(lca_probe_hbm_read(nullptr, 1024, static_cast<uint32_t *>(A), nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_hbm_read(A, 1024, nullptr, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_hbm_read(A, 0, static_cast<uint32_t *>(A), nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_hbm_read(A, 1000, static_cast<uint32_t *>(A), nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_hbm_read(odd, 1024, static_cast<uint32_t *>(A), nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_mfma_bf16(0, 0, static_cast<float *>(A), &waves, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_mfma_bf16(65537, 1, static_cast<float *>(A), &waves, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_mfma_bf16(16, 2, static_cast<float *>(A), &waves, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_mfma_bf16(16, 0, nullptr, &waves, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(lca_probe_mfma_bf16(16, 0, static_cast<float *>(A), nullptr, nullptr) == LCA_ERR_INVALID_ARG);
    EXPECT(waves == -7);
    std::printf("checks %d failed %d\n", n_checks, n_bad);
    return n_bad == 0 ? 0 : 1;
}
