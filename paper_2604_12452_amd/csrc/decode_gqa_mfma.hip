// Decode step over a condensed cache at the GQA widths (d_k = d_v = 128, bf16 or fp16; section 4.3 of the paper,
// decoding paragraph, with the GQA form of section 5.4: hard-selected keys, pooled values per KV head) on the
// matrix cores.  The vector-ALU kernel of decode.hip spends ~25 instructions per cache row and query head and is
// compute-bound from five heads per KV head on; here the (up to 16) query heads of a KV head are the 16 columns of
// 16x16x32 MFMAs, as in the MLA decode kernel:
//   S^T[key, head]  = K Q^T       A = 16 key rows from LDS (16-byte reads), B = Q^T in registers (4 k-steps)
//   O^T[dv, head]  += V^T P^T     A = V^T through LDS transpose reads,       B = P^T = exp2(S^T - ref)
// Every WAVEFRONT works alone on its own range of entries (no barriers in the loop) with two 16 KB tile buffers of
// its own: a tile is 32 entries, keys 32 x 256 B and values 32 x 256 B, copied with direct-to-LDS loads of four rows
// each; the copy of tile t+1 is in flight while tile t is used.  Rows are 256 B apart, so instead of padding the
// 16-byte chunk c of row r sits at slot c ^ (r mod 16): the copy permutes the chunks on the global side, and both
// the key reads (16 rows, one chunk each) and the transpose reads (rows 4 apart) are conflict-free.  S^T row m of a
// block of 16 comes from LDS row 4(m%4) + m/4, so that the S^T accumulators already are the B fragments of the
// second product.  Softmax keeps one fixed reference per head (taken at the first tile); if a row sum ends beyond
// 2^100 (or, in fp16, an exponential left the type's range and the sum is infinite) the wavefront collects the
// exact maximum of its range and runs it again.  The four wavefronts' results are merged in LDS into one partial
// result per workgroup; the workgroups' partial results are merged by decode_merge_kernel.
#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4 mfma_16x16x32(bf16x8 a, bf16x8 b, floatx4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ floatx4 mfma_16x16x32(f16x8 a, f16x8 b, floatx4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ bf16x4 lds_read_tr16(__attribute__((address_space(3))) bf16x4 *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(p); }
__device__ __forceinline__ f16x4 lds_read_tr16(__attribute__((address_space(3))) f16x4 *p)
{
    typedef __fp16 fp16x4 __attribute__((__vector_size__(4 * sizeof(__fp16))));     // the builtin's own spelling of four halves
    return __builtin_bit_cast(f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4f16((__attribute__((address_space(3))) fp16x4 *)p));
}

constexpr int D = 128;
constexpr int BN = 32;                          // entries per tile
constexpr int RB = D * 2;                       // bytes per row
constexpr int V_OFF = BN * RB;                  // the value rows of a tile follow its key rows
constexpr int TILE_BYTES = 2 * BN * RB;         // 16 KB
constexpr int NKS = D / 32;                     // 4 k-steps of S^T
constexpr int NDT = D / 16;                     // 8 value tiles
constexpr int COPIES = 2 * BN / 4;              // direct-to-LDS loads per tile (four rows each): 16
constexpr int MROW = D + 4;                     // floats per head of a wavefront's rescaled output in LDS (merge at the end)
static_assert(16 * MROW * 4 <= 2 * TILE_BYTES, "the rescaled output of 16 heads fits a wavefront's tile buffers");
constexpr float NEG_BIG = -1.0e30f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float SUM_LIMIT = 0x1p100f;

struct DgParams {
    const uint16_t *q, *k_rep, *v_rep, *k_tail, *v_tail;
    const uint8_t *k_q8, *v_q8;            // 8-bit representatives (E4M3 codes) and their row scales [.., m_cap, 2] = (value, key), or NULL
    const float *scales;
    float *part;
    void *O;                               // not NULL: one workgroup per (sequence, KV head), which then writes the final output itself
    int S, hps, m, k, n_parts, m_cap, k_cap, k_start;
    float scale_log2, bias_log2;
};

__device__ __forceinline__ unsigned lds_address(const char *p) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p; }

// Direct-to-LDS load of 64 x 16 bytes from per-lane addresses (lane l -> LDS [lds_addr + 16 l, +16)); inline assembly
// so that the compiler does not tie later LDS reads to it -- the wavefront waits for its copies by hand.
__device__ __forceinline__ void dma_lanes(const void *addr, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(addr), "s"(lds_addr));
}

// Two E4M3 codes (the low or the high half of w) times a power-of-two scale, as two elements of type E: exact.
template <typename E> __device__ __forceinline__ unsigned cvt2_fp8(unsigned w, float scale, bool high);
template <> __device__ __forceinline__ unsigned cvt2_fp8<__bf16>(unsigned w, float scale, bool high)
{
    return high ? __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, scale, true))
                : __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, scale, false));
}
template <> __device__ __forceinline__ unsigned cvt2_fp8<_Float16>(unsigned w, float scale, bool high)
{
    return high ? __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, scale, true))
                : __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, scale, false));
}
template <typename E> __device__ __forceinline__ void cvt16_fp8(const uint4 &c, float scale, uint4 &lo, uint4 &hi)
{
    lo = make_uint4(cvt2_fp8<E>(c.x, scale, false), cvt2_fp8<E>(c.x, scale, true), cvt2_fp8<E>(c.y, scale, false), cvt2_fp8<E>(c.y, scale, true));
    hi = make_uint4(cvt2_fp8<E>(c.z, scale, false), cvt2_fp8<E>(c.z, scale, true), cvt2_fp8<E>(c.w, scale, false), cvt2_fp8<E>(c.w, scale, true));
}

// Q8: the representatives come as E4M3 codes with a power-of-two scale per row and component.  A tile then holds
// entries of one kind only (the list of tiles is the representatives' tiles followed by the tail's), and a tile of
// representatives (4 KB of key codes, 4 KB of value codes, contiguous) is fetched into registers while the tile before it
// is used, converted -- one instruction per two codes, the row's scale riding along -- and written into the LDS
// layout of the 16-bit tiles; from there on nothing differs.
template <typename E, bool Q8>
__global__ __launch_bounds__(256, 1) void decode_gqa_mfma_kernel(const DgParams kp)
{
    typedef E ex8 __attribute__((ext_vector_type(8)));
    typedef E ex4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(1024))) char bufs[4][2][TILE_BYTES];
    __shared__ float wave_ml[4][16][2];                                     // (reference, sum) per wavefront and head
    __shared__ float l_heads[16];                                           // merged sum per head

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 15, q4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg_per_bs = kp.n_parts / 4;
    const int part = (blockIdx.x % wg_per_bs) * 4 + wave, bs = blockIdx.x / wg_per_bs;
    const int m = kp.m, n = kp.m + kp.k;
    const int rep_tiles = Q8 ? (m + BN - 1) / BN : 0;                       // Q8: tiles [0, rep_tiles) hold representatives only
    const int tiles_total = Q8 ? rep_tiles + (kp.k + BN - 1) / BN : (n + BN - 1) / BN;
    const int tiles_per_part = (tiles_total + kp.n_parts - 1) / kp.n_parts;
    const int t_lo = min(part * tiles_per_part, tiles_total), t_hi = min(t_lo + tiles_per_part, tiles_total);
    const int e_hi = Q8 ? n : min(n, t_hi * BN);
    // first entry of tile tl and the end of the entries it may show (Q8: the end of its kind)
    auto is_q8 = [&](int tl) { return Q8 && tl < rep_tiles; };
    auto first_entry = [&](int tl) { return !Q8 ? tl * BN : tl < rep_tiles ? tl * BN : m + (tl - rep_tiles) * BN; };
    auto segment_end = [&](int tl) { return !Q8 ? e_hi : tl < rep_tiles ? m : n; };
    char *buf0 = bufs[wave][0];
    const unsigned buf_lds = lds_address(buf0);

    // source rows: entry e < m is representative e, else tail token e - m in ring row (k_start + e - m) mod k_cap
    const uint16_t *krep = kp.k_rep + (size_t)bs * kp.m_cap * D, *vrep = kp.v_rep + (size_t)bs * kp.m_cap * D;
    const uint16_t *ktail = kp.k_tail + (size_t)bs * kp.k_cap * D, *vtail = kp.v_tail + (size_t)bs * kp.k_cap * D;

    ex8 qf[NKS];        // Q^T fragments, loaded below once the first tile's copy is on its way

    // per-lane LDS offsets inside a tile buffer: chunk c (16 bytes) of row r sits at slot c ^ (r & 15)
    const int krow = 4 * (col & 3) + (col >> 2);                            // LDS row behind S^T row `col` of a block of 16
    int k_off[NKS];                                                         // + 16*blk*RB
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_off[ks] = krow * RB + (((4 * ks + q4) ^ krow) << 4);
    const int vrow = 4 * (col >> 2) + q4;                                   // transpose read of 4 keys (rows 4 apart) x 4 columns
    const int v_base = V_OFF + vrow * RB + 8 * (col & 1), v_c1 = (col >> 1) & 1;   // + 16*hh*RB, chunk 2t + v_c1 at slot ^ vrow

    floatx4 acc[NDT];
    float m_ref = NEG_BIG, l_run = 0.f, m_seen = NEG_BIG;
    const float c = kp.scale_log2;
    typedef __attribute__((address_space(3))) ex4 *lds_b64_ptr;

    // copy of tile tl into tile buffer `b`: load i brings rows 4i .. 4i+3 of the keys (i < 8) or of the values; lane l
    // fills slot l & 15 of row 4i + (l >> 4), i.e. fetches chunk (l & 15) ^ (row & 15); rows past the range repeat its last row
    auto issue_copy = [&](int tl, int b) {
        const int e0 = first_entry(tl), seg_end = segment_end(tl);
#pragma unroll
        for (int i = 0; i < BN / 4; ++i) {
            const int r = 4 * i + (lane >> 4);
            const int e = min(e0 + r, seg_end - 1);
            int t = kp.k_start + e - m;
            t = t >= kp.k_cap ? t - kp.k_cap : t;
            const size_t off = (e < m ? (size_t)e : (size_t)t) * D + (((lane & 15) ^ (r & 15)) << 3);
            dma_lanes((e < m ? krep : ktail) + off, buf_lds + b * TILE_BYTES + 4 * i * RB);
            dma_lanes((e < m ? vrep : vtail) + off, buf_lds + b * TILE_BYTES + V_OFF + 4 * i * RB);
        }
    };

    // Q8: the codes of one tile of representatives in registers.  Load i (of 4 for the keys, 4 for the values) brings rows
    // 8i .. 8i+7 (lane l: 16 codes at column 16 (l & 7) of row 8i + (l >> 3)); lane r < 32 holds the two scales of row r.
    // Rows past the end repeat the last one.
    uint4 q8_k[BN / 8], q8_v[BN / 8];
    float2 q8_scale = float2{1.f, 1.f};
    auto fetch_q8 = [&](int tl) {
        const uint8_t *kq = kp.k_q8 + (size_t)bs * kp.m_cap * D, *vq = kp.v_q8 + (size_t)bs * kp.m_cap * D;
        const int e0 = tl * BN;
#pragma unroll
        for (int i = 0; i < BN / 8; ++i) {
            const size_t off = (size_t)min(e0 + 8 * i + (lane >> 3), m - 1) * D + 16 * (lane & 7);
            q8_k[i] = *reinterpret_cast<const uint4 *>(kq + off);
            q8_v[i] = *reinterpret_cast<const uint4 *>(vq + off);
        }
        q8_scale = *reinterpret_cast<const float2 *>(kp.scales + ((size_t)bs * kp.m_cap + min(e0 + (lane & 31), m - 1)) * 2);
    };
    // ... converted (the row's scale riding along) and written in the 16-bit layout: chunk c of row r at slot c ^ (r & 15)
    auto convert_q8 = [&](char *buf) {
#pragma unroll
        for (int i = 0; i < BN / 8; ++i) {
            const int r = 8 * i + (lane >> 3), c0 = 2 * (lane & 7);
            const float sv = __shfl(q8_scale.x, r, 64), sk = __shfl(q8_scale.y, r, 64);
            uint4 lo, hi;
            cvt16_fp8<E>(q8_k[i], sk, lo, hi);
            *reinterpret_cast<uint4 *>(buf + r * RB + ((c0 ^ (r & 15)) << 4)) = lo;
            *reinterpret_cast<uint4 *>(buf + r * RB + (((c0 + 1) ^ (r & 15)) << 4)) = hi;
            cvt16_fp8<E>(q8_v[i], sv, lo, hi);
            *reinterpret_cast<uint4 *>(buf + V_OFF + r * RB + ((c0 ^ (r & 15)) << 4)) = lo;
            *reinterpret_cast<uint4 *>(buf + V_OFF + r * RB + (((c0 + 1) ^ (r & 15)) << 4)) = hi;
        }
    };
    auto issue = [&](int tl, int b) {
        if (is_q8(tl)) fetch_q8(tl);
        else issue_copy(tl, b);
    };

    // S^T = K Q^T for the two blocks of 16 entries of the tile in `buf`, and the logits in base 2 (scale, bias of the
    // representatives, entries past the range hidden)
    auto tile_logits = [&](int tl, const char *buf, float (&lg)[2][4]) {
        const int e0 = first_entry(tl), seg_end = segment_end(tl);
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            ex8 kf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) kf[ks] = *reinterpret_cast<const ex8 *>(buf + blk * 16 * RB + k_off[ks]);
            floatx4 sacc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) sacc = mfma_16x16x32(kf[ks], qf[ks], sacc);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = e0 + blk * 16 + 4 * r + q4;                   // accumulator row 4 q4 + r sits in LDS row 4 r + q4
                lg[blk][r] = e < seg_end ? fmaf(sacc[r], c, e < m ? kp.bias_log2 : 0.f) : -INFINITY;
            }
        }
    };
    auto head_max = [&](const float (&lg)[2][4]) {
        float mx = NEG_BIG;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, lg[blk][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        return fmaxf(mx, __shfl_xor(mx, 32, 64));
    };
    // (the queries travel together with the first tile: their latency is paid once, not before the first copy starts)
    bool q_loaded = false;
    auto load_q = [&]() {
        // Q^T fragments: lane (col = head of the KV head, q4) holds q[head, 32 ks + 8 q4 .. +7]; columns past the heads are zero
        {
            const uint16_t *qp = kp.q + ((size_t)bs * kp.hps + min(col, kp.hps - 1)) * D + 8 * q4;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                qf[ks] = *reinterpret_cast<const ex8 *>(qp + 32 * ks);
                if (col >= kp.hps) qf[ks] = ex8{0, 0, 0, 0, 0, 0, 0, 0};
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) asm volatile("" : "+v"(qf[ks]));   // here before the loop starts (its waits count copies)
        }
        q_loaded = true;
    };
    // One sweep over the wavefront's tiles.  Tile tl sits in buffer (tl - t_lo) & 1; tile tl+1 is on its way -- by direct-to-LDS
    // copy into the other buffer, or into the registers -- while `body` uses tile tl.  (A tile of codes is never followed
    // by one before it in kind, so behind the copies of a 16-bit tile only copies of a 16-bit tile can be in flight.)
    auto sweep = [&](auto &&body) {
        if (t_lo < t_hi) issue(t_lo, 0);
        if (!q_loaded) load_q();
        for (int tl = t_lo; tl < t_hi; ++tl) {
            const int b = (tl - t_lo) & 1;
            char *buf = buf0 + b * TILE_BYTES;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");              // this wavefront's reads of tile tl-1 (and tl-2) are done
            if (is_q8(tl)) {
                convert_q8(buf);
                if (tl + 1 < t_hi) issue(tl + 1, b ^ 1);
            } else if (tl + 1 < t_hi) {
                issue_copy(tl + 1, b ^ 1);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(COPIES) : "memory");   // tile tl has landed, tile tl+1 may still travel
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            body(tl, buf);
        }
    };

    float l_tot = 0.f;
    for (bool again = false;;) {                                            // normally one pass; a second one from the exact maxima
#pragma unroll
        for (int t = 0; t < NDT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        l_run = 0.f;
        m_ref = again ? m_seen : NEG_BIG;
        bool ref_missing = !again;

        sweep([&](int tl, const char *buf) {
            float lg[2][4];
            tile_logits(tl, buf, lg);
            if (ref_missing) {                                              // the first tile fixes the reference
                const float mx = head_max(lg);
                m_ref = (m_ref == NEG_BIG) ? mx : m_ref;
                ref_missing = __builtin_amdgcn_ballot_w64(m_ref == NEG_BIG) != 0;
            }
            // P^T in the element type (B fragment: k-slot i < 4 is the key of block 0 register i, i >= 4 of block 1 register
            // i-4) and its sum (of the rounded values, the ones the second product sees)
            ex8 pb;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pb[blk * 4 + r] = (E)__builtin_amdgcn_exp2f(lg[blk][r] - m_ref);
                    l_run += (float)pb[blk * 4 + r];
                }
            // O^T += V^T P^T over the 8 value tiles
            ex4 vlo[NDT], vhi[NDT];
#pragma unroll
            for (int t = 0; t < NDT; ++t) {
                const char *vp = buf + v_base + (((2 * t + v_c1) ^ vrow) << 4);
                vlo[t] = lds_read_tr16((lds_b64_ptr)(vp));
                vhi[t] = lds_read_tr16((lds_b64_ptr)(vp + 16 * RB));
            }
#pragma unroll
            for (int t = 0; t < NDT; ++t) {
                const ex8 a = __builtin_shufflevector(vlo[t], vhi[t], 0, 1, 2, 3, 4, 5, 6, 7);
                acc[t] = mfma_16x16x32(a, pb, acc[t]);
            }
        });

        l_tot = l_run + __shfl_xor(l_run, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        if (again || __builtin_amdgcn_ballot_w64(!(l_tot <= SUM_LIMIT)) == 0) break;
        // (wave-uniform) a head ran out of exponent headroom: exact maxima of the range, then the pass again
        m_seen = NEG_BIG;
        sweep([&](int tl, const char *buf) {
            float lg[2][4];
            tile_logits(tl, buf, lg);
            m_seen = fmaxf(m_seen, head_max(lg));
        });
        again = true;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                      // the last tile's reads are done before the buffers are reused

    // The four wavefronts' results (reference, sum, unnormalised output per head) are merged here, through LDS, so that
    // one partial result per workgroup goes to memory: each wavefront publishes its references and sums, rescales its
    // accumulators to the common reference into its own (now idle) tile buffers, and then adds up a quarter of the
    // value columns over the four wavefronts' buffers.
    const bool any = t_lo < t_hi;
    if (q4 == 0) {
        wave_ml[wave][col][0] = any ? m_ref : -INFINITY;
        wave_ml[wave][col][1] = any ? l_tot : 0.f;
    }
    __syncthreads();
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, wave_ml[w][col][0]);
    float l_all = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float mw = wave_ml[w][col][0];
        l_all += mw == -INFINITY ? 0.f : wave_ml[w][col][1] * __builtin_amdgcn_exp2f(mw - m_all);
    }
    {
        const float f = any ? __builtin_amdgcn_exp2f(m_ref - m_all) : 0.f;
        float *mine = reinterpret_cast<float *>(buf0) + col * MROW + 4 * q4;   // [head][MROW] floats
#pragma unroll
        for (int t = 0; t < NDT; ++t) {
            floatx4 v = acc[t];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = any ? v[r] * f : 0.f;
            *reinterpret_cast<floatx4 *>(mine + 16 * t) = v;
        }
    }
    if (wave == 0 && q4 == 0) l_heads[col] = l_all;
    __syncthreads();
    // wavefront w adds up value columns [32 w, 32 w + 32) of every head (lane l: head l >> 5 + 2 j in step j, column
    // 32 w + (l & 31)) and writes them: as this workgroup's partial result (natural-log units), or -- when the workgroup
    // has the whole (sequence, KV head) to itself -- normalised, as the final output
    float *dst0 = kp.part + ((size_t)bs * wg_per_bs + blockIdx.x % wg_per_bs) * kp.hps * (D + 2);
    for (int h = lane >> 5; h < kp.hps; h += 2) {
        const int x = 32 * wave + (lane & 31);
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) sum += reinterpret_cast<const float *>(bufs[w][0])[h * MROW + x];
        if (kp.O != nullptr) reinterpret_cast<E *>(kp.O)[((size_t)bs * kp.hps + h) * D + x] = (E)(sum / l_heads[h]);
        else dst0[(size_t)h * (D + 2) + 2 + x] = sum;
    }
    if (kp.O != nullptr) return;
    if (wave == 0 && q4 == 0 && col < kp.hps) {
        float *dst = dst0 + (size_t)col * (D + 2);
        dst[0] = m_all == -INFINITY ? -INFINITY : m_all * LN2;
        dst[1] = l_all;
    }
}

}  // namespace

bool decode_gqa_mfma_supported(const Dims &d)
{
    const int hps = d.H / d.S;
    return (d.dtype == LCA_BF16 || d.dtype == LCA_F16) && d.mode == LCA_MODE_GQA && d.d_pool == D && d.d_sel == D && hps <= 16 && d.scale > 0.f;
}

// partial results per (sequence, KV head): a multiple of 4 (one per wavefront), enough workgroups to fill the chip, at
// least four tiles per wavefront where the cache is long enough
int decode_gqa_mfma_parts(const Dims &d)
{
    const int tiles = (d.m + BN - 1) / BN + (d.k + BN - 1) / BN;      // (an upper bound when the two kinds share tiles)
    int wgs = (256 + d.B * d.S - 1) / (d.B * d.S);
    const int max_wgs = (tiles + 15) / 16;
    if (wgs > max_wgs) wgs = max_wgs;
    if (wgs < 1) wgs = 1;
    return 4 * wgs;
}

hipError_t launch_decode_gqa_mfma(const DecodeArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    DgParams kp;
    kp.q = (const uint16_t *)a.q; kp.k_rep = (const uint16_t *)a.sel_rep; kp.v_rep = (const uint16_t *)a.pool_rep;
    kp.k_tail = (const uint16_t *)a.sel_tail; kp.v_tail = (const uint16_t *)a.pool_tail; kp.part = a.part;
    kp.S = d.S; kp.hps = d.H / d.S; kp.m = d.m; kp.k = d.k; kp.n_parts = a.splits;
    kp.m_cap = a.m_cap; kp.k_cap = a.k_cap; kp.k_start = a.k_start;
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    kp.k_q8 = a.sel_q8; kp.v_q8 = a.pool_q8; kp.scales = a.scales;
    kp.O = a.splits == 4 ? a.O : nullptr;
    const unsigned grid = d.B * d.S * (a.splits / 4);
    if (a.pool_q8 != nullptr) {
        if (d.dtype == LCA_F16) decode_gqa_mfma_kernel<_Float16, true><<<grid, 256, 0, st>>>(kp);
        else decode_gqa_mfma_kernel<__bf16, true><<<grid, 256, 0, st>>>(kp);
    } else {
        if (d.dtype == LCA_F16) decode_gqa_mfma_kernel<_Float16, false><<<grid, 256, 0, st>>>(kp);
        else decode_gqa_mfma_kernel<__bf16, false><<<grid, 256, 0, st>>>(kp);
    }
    return hipGetLastError();
}

}  // namespace lca
