// Decode step over a condensed cache at the MLA widths (d_c = 512, d_R = 64, bf16 or fp16; section 4.3 of the paper,
// decoding paragraph; absorbed form of section 3): the new token's query attends the m representatives and the
// k raw tail rows, and the (up to 16) heads of a condensed set share every cache row.
//
// One cache row of 1152 bytes feeds 16 heads x (576 + 512) multiply-adds, about 30 flops per byte: at HBM speed
// that is beyond the vector ALU, so the products run on the matrix cores with the heads as the 16 columns of
// 16x16x32 MFMAs:
//   S^T[key, head]  = K Q^T       A = 16 key rows from LDS (16-byte reads), B = Q^T in registers (18 k-steps)
//   O^T[dv, head]  += V^T P^T     A = V^T through LDS transpose reads,       B = P^T = exp2(S^T - ref)
// Every WAVEFRONT works alone on its own range of entries (no barriers in the loop) with two 18 KB LDS buffers of its
// own: a tile is 16 entries (16 latent rows of 1 KB at a 1040-byte stride, the RoPE parts XOR-swizzled), copied with
// direct-to-LDS loads; the copy of tile t+1 is in flight while tile t is used -- twice: all 576 columns as keys, the
// first 512 as values.  S^T row m of the tile comes from LDS row 4(m%4) + m/4, so that the S^T accumulators already
// are the B fragments of the second product (16x16x16 MFMAs) when the transpose reads of a 16-lane block take rows 4
// apart (conflict-free on the 1040-byte stride).  Softmax keeps one fixed reference per head (taken at the first
// tile), so the 128 accumulation registers are never rescaled; if a row sum ends beyond 2^100 (or, in fp16, an
// exponential left the type's range and the sum is infinite) the wavefront collects the exact maximum of its range
// and runs it again.  The four wavefronts' results (reference, sum, unnormalised output per head) are merged in LDS
// into one partial result per workgroup; the workgroups' partial results are merged by decode_merge_kernel.
#include "lca_internal.h"
#include "mla_tile16.h"

namespace lca {
namespace {

using namespace tile16;

// A row sum beyond this (or not finite) makes the wavefront run its range again from the exact maxima.  The sum adds the
// ROUNDED exponentials, so one that left fp16's range (65504) arrives here as an infinity.
constexpr float SUM_LIMIT = 0x1p100f;

constexpr int NKS = DQK / 32;                   // 18 k-steps of S^T
constexpr int NDT = DP / 16;                    // 32 value tiles
constexpr int PV_GROUP = 8;                     // value tiles whose V^T fragments are requested together
constexpr int MROW = DP + 4;                    // floats per head of a wavefront's rescaled output in LDS (merge at the end)
static_assert(16 * MROW * 4 <= 2 * BUF_BYTES, "the rescaled output of 16 heads fits a wavefront's two tile buffers");
constexpr float NEG_BIG = -1.0e30f;
constexpr float LN2 = 0.6931471805599453f;

struct DmParams {
    const uint16_t *q, *pool_rep, *sel_rep, *pool_tail, *sel_tail;
    const uint8_t *pool_q8, *sel_q8;       // 8-bit representatives (E4M3 codes) and their row scales [.., m_cap, 2], or NULL
    const float *scales;
    float *part;
    void *O;                               // not NULL: one workgroup per (sequence, set), which then writes the final output itself
    int S, hps, m, k, n_parts, m_cap, k_cap, k_start;
    float scale_log2, bias_log2;
};

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
// 16 codes -> 16 elements (two 16-byte pieces)
template <typename E> __device__ __forceinline__ void cvt16_fp8(const uint4 &c, float scale, uint4 &lo, uint4 &hi)
{
    lo = make_uint4(cvt2_fp8<E>(c.x, scale, false), cvt2_fp8<E>(c.x, scale, true), cvt2_fp8<E>(c.y, scale, false), cvt2_fp8<E>(c.y, scale, true));
    hi = make_uint4(cvt2_fp8<E>(c.z, scale, false), cvt2_fp8<E>(c.z, scale, true), cvt2_fp8<E>(c.w, scale, false), cvt2_fp8<E>(c.w, scale, true));
}

// Q8: the representatives come as E4M3 codes with a power-of-two scale per row and component.  A tile then holds
// entries of one kind only (the list of tiles is the representatives' tiles followed by the tail's), and a tile of
// representatives is fetched into registers (its 8 KB + 1 KB of codes are contiguous) while the tile before it is used,
// converted -- one instruction per two codes, the row's scale riding along -- and written into the same LDS layout
// the 16-bit tiles use; from there on nothing differs.
template <typename E, bool Q8>
__global__ __launch_bounds__(256, 1) void decode_mla_kernel(const DmParams kp)
{
    typedef E ex8 __attribute__((ext_vector_type(8)));
    typedef E ex4 __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(1024))) char bufs[4][2][BUF_BYTES];
    __shared__ float wave_ml[4][16][2];                                     // (reference, sum) per wavefront and head
    __shared__ float l_heads[16];                                           // merged sum per head

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 15, q4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg_per_bs = kp.n_parts / 4;
    const int part = (blockIdx.x % wg_per_bs) * 4 + wave, bs = blockIdx.x / wg_per_bs;
    const int b = bs / kp.S;
    const int m = kp.m, n = kp.m + kp.k;
    const int rep_tiles = Q8 ? (m + BN - 1) / BN : 0;                       // Q8: tiles [0, rep_tiles) hold representatives only
    const int tiles_total = Q8 ? rep_tiles + (kp.k + BN - 1) / BN : (n + BN - 1) / BN;
    const int tiles_per_part = (tiles_total + kp.n_parts - 1) / kp.n_parts;
    const int t_lo = min(part * tiles_per_part, tiles_total), t_hi = min(t_lo + tiles_per_part, tiles_total);
    const int e_hi = Q8 ? n : min(n, t_hi * BN);
    char *buf0 = bufs[wave][0];
    const unsigned buf_lds = lds_address(buf0);

    // source rows: entry e < m is representative e, else tail token e - m in ring row (k_start + e - m) mod k_cap
    const uint16_t *prep = kp.pool_rep + (size_t)bs * kp.m_cap * DP, *srep = kp.sel_rep + (size_t)bs * kp.m_cap * DS;
    const uint16_t *ptail = kp.pool_tail + (size_t)b * kp.k_cap * DP, *stail = kp.sel_tail + (size_t)b * kp.k_cap * DS;
    auto ring_row = [&](int e) { const int t = kp.k_start + e - m; return t >= kp.k_cap ? t - kp.k_cap : t; };
    // first entry of tile tl and the end of the entries it may show (Q8: the end of its kind)
    auto is_q8 = [&](int tl) { return Q8 && tl < rep_tiles; };
    auto first_entry = [&](int tl) { return !Q8 ? tl * BN : tl < rep_tiles ? tl * BN : m + (tl - rep_tiles) * BN; };
    auto segment_end = [&](int tl) { return !Q8 ? e_hi : tl < rep_tiles ? m : n; };

    ex8 qf[NKS];        // Q^T fragments, loaded below once the first tile's copy is on its way

    // per-lane LDS offsets inside a tile buffer
    const int krow = 4 * (col & 3) + (col >> 2);                            // LDS row behind S^T row `col` of the tile's 16 entries
    const int k_off = krow * RSB + 16 * q4;                                 // + 64*ks
    const int ksel_row = SEL_OFF + krow * (DS * 2);                         // chunk c at slot c ^ (row & 7)
    const int v_off = (4 * (col >> 2) + q4) * RSB + 8 * (col & 3);          // + 32*t: transpose read of 4 keys (rows 4 apart) x 4 columns

    floatx4 acc[NDT];
    float m_ref = NEG_BIG, l_run = 0.f, m_seen = NEG_BIG;
    const float c = kp.scale_log2;
    typedef __attribute__((address_space(3))) ex4 *lds_b64_ptr;

    // Q8: the codes of one tile of representatives in registers.  Load i brings rows 2i, 2i+1 of the latent part (lane l:
    // 16 codes at column 16 (l & 31) of row 2i + (l >> 5)), one more the RoPE part (lane l: 16 codes at column 16 (l & 3)
    // of row l >> 2); lane r < 16 holds the two scales of row r.  Rows past the end repeat the last one.
    uint4 q8_pool[BN / 2], q8_sel;
    float2 q8_scale = float2{1.f, 1.f};
    auto fetch_q8 = [&](int tl) {
        const uint8_t *pq = kp.pool_q8 + (size_t)bs * kp.m_cap * DP, *sq = kp.sel_q8 + (size_t)bs * kp.m_cap * DS;
        const int e0 = tl * BN;
#pragma unroll
        for (int i = 0; i < BN / 2; ++i) {
            const int e = min(e0 + 2 * i + (lane >> 5), m - 1);
            q8_pool[i] = *reinterpret_cast<const uint4 *>(pq + (size_t)e * DP + 16 * (lane & 31));
        }
        q8_sel = *reinterpret_cast<const uint4 *>(sq + (size_t)min(e0 + (lane >> 2), m - 1) * DS + 16 * (lane & 3));
        q8_scale = *reinterpret_cast<const float2 *>(kp.scales + ((size_t)bs * kp.m_cap + min(e0 + (lane & 15), m - 1)) * 2);
    };
    // ... converted (one instruction per two codes, the row's scale riding along) and written in the 16-bit layout
    auto convert_q8 = [&](char *buf) {
#pragma unroll
        for (int i = 0; i < BN / 2; ++i) {
            const float s0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, q8_scale.x), 2 * i));
            const float s1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, q8_scale.x), 2 * i + 1));
            uint4 lo, hi;
            cvt16_fp8<E>(q8_pool[i], lane < 32 ? s0 : s1, lo, hi);
            char *dst = buf + (2 * i + (lane >> 5)) * RSB + 32 * (lane & 31);
            *reinterpret_cast<uint4 *>(dst) = lo;
            *reinterpret_cast<uint4 *>(dst + 16) = hi;
        }
        const int r = lane >> 2, c0 = 2 * (lane & 3);                       // chunk c of row r sits at slot c ^ (r & 7)
        uint4 lo, hi;
        cvt16_fp8<E>(q8_sel, __shfl(q8_scale.y, r, 64), lo, hi);
        char *dst = buf + SEL_OFF + r * (DS * 2);
        *reinterpret_cast<uint4 *>(dst + ((c0 ^ (r & 7)) << 4)) = lo;
        *reinterpret_cast<uint4 *>(dst + (((c0 + 1) ^ (r & 7)) << 4)) = hi;
    };
    // 16-bit tiles: COPIES direct-to-LDS loads into tile buffer `bi` -- 16 latent rows (one load each) and the RoPE parts
    // of 8 rows per load; rows past the range repeat its last row
    auto issue_dma = [&](int tl, int bi) {
        const int e0 = first_entry(tl), seg_end = segment_end(tl), e_last = e0 + BN - 1;
        const unsigned dst = buf_lds + bi * BUF_BYTES;
        // the usual tile: 16 consecutive rows of one buffer (no end of range, no rep/tail seam, no wrap of the ring)
        const bool in_rep = e_last < m, in_tail = e0 >= m && ring_row(e0) + BN <= kp.k_cap;
        if (e_last < seg_end && (in_rep || in_tail)) {
            const size_t row0 = in_rep ? e0 : ring_row(e0);
            const char *pb0 = (const char *)((in_rep ? prep : ptail) + row0 * DP);
            const char *sb0 = (const char *)((in_rep ? srep : stail) + row0 * DS);
#pragma unroll
            for (int r = 0; r < BN; ++r) dma_row(lane * 16, pb0 + r * (DP * 2), dst + r * RSB);
#pragma unroll
            for (int j = 0; j < BN / 8; ++j) {
                const int r = 8 * j + (lane >> 3);
                dma_row(r * (DS * 2) + (((lane & 7) ^ (r & 7)) << 4), sb0, dst + SEL_OFF + 8 * j * (DS * 2));
            }
        } else {
#pragma unroll 4
            for (int r = 0; r < BN; ++r) {
                const int e = min(e0 + r, seg_end - 1);
                const uint16_t *src = e < m ? prep + (size_t)e * DP : ptail + (size_t)ring_row(e) * DP;
                dma_row(lane * 16, src, dst + r * RSB);
            }
#pragma unroll
            for (int j = 0; j < BN / 8; ++j) {
                const int r = 8 * j + (lane >> 3);
                const int e = min(e0 + r, seg_end - 1);
                const uint16_t *src = (e < m ? srep + (size_t)e * DS : stail + (size_t)ring_row(e) * DS) + (((lane & 7) ^ (r & 7)) << 3);
                dma_lanes(src, dst + SEL_OFF + 8 * j * (DS * 2));
            }
        }
    };
    auto issue = [&](int tl, int bi) {
        if (is_q8(tl)) fetch_q8(tl);
        else issue_dma(tl, bi);
    };
    // (the queries travel together with the first tile: their latency is paid once, not before the first copy starts)
    bool q_loaded = false;
    auto load_q = [&]() {
        // Q^T fragments: lane (col = head of the set, q4) holds q[head, 32 ks + 8 q4 .. +7]; columns past the set's heads are zero
        {
            const uint16_t *qp = kp.q + ((size_t)bs * kp.hps + min(col, kp.hps - 1)) * DQK + 8 * q4;
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
            const int bi = (tl - t_lo) & 1;
            char *buf = buf0 + bi * BUF_BYTES;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");              // this wavefront's reads of tile tl-1 (and tl-2) are done
            if (is_q8(tl)) {
                convert_q8(buf);
                if (tl + 1 < t_hi) issue(tl + 1, bi ^ 1);
            } else if (tl + 1 < t_hi) {
                issue_dma(tl + 1, bi ^ 1);
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(COPIES) : "memory");   // tile tl has landed, tile tl+1 may still travel
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            body(tl, buf);
        }
    };
    // S^T = K Q^T for the tile's 16 entries, and the logits in base 2 (scale, bias of the representatives, entries past the
    // range hidden): accumulator register r of this lane is entry 4 r + q4 of the tile
    auto tile_logits = [&](int tl, const char *buf, float (&lg)[4]) {
        const int e0 = first_entry(tl), seg_end = segment_end(tl);
        ex8 kf[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const char *p = ks < DP / 32 ? buf + k_off + 64 * ks : buf + ksel_row + (((4 * (ks - DP / 32) + q4) ^ (krow & 7)) << 4);
            kf[ks] = *reinterpret_cast<const ex8 *>(p);
        }
        __builtin_amdgcn_sched_barrier(0);
        floatx4 sacc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) sacc = mfma_16x16x32(kf[ks], qf[ks], sacc);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e = e0 + 4 * r + q4;                                  // accumulator row 4 q4 + r sits in LDS row 4 r + q4
            lg[r] = e < seg_end ? fmaf(sacc[r], c, e < m ? kp.bias_log2 : 0.f) : -INFINITY;
        }
    };
    auto head_max = [&](const float (&lg)[4]) {
        float mx = fmaxf(fmaxf(fmaxf(lg[0], lg[1]), fmaxf(lg[2], lg[3])), NEG_BIG);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        return fmaxf(mx, __shfl_xor(mx, 32, 64));
    };

    float l_tot = 0.f;
    for (bool again = false;;) {                                            // normally one pass; a second one from the exact maxima
#pragma unroll
        for (int t = 0; t < NDT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        l_run = 0.f;
        m_ref = again ? m_seen : NEG_BIG;
        bool ref_missing = !again;

        sweep([&](int tl, const char *buf) {
            float lg[4];
            tile_logits(tl, buf, lg);
            if (ref_missing) {                                              // the first tile fixes the reference
                const float mx = head_max(lg);
                m_ref = (m_ref == NEG_BIG) ? mx : m_ref;
                ref_missing = __builtin_amdgcn_ballot_w64(m_ref == NEG_BIG) != 0;
            }
            // P^T in the element type (B fragment of a 16x16x16 product: k-slot r of this lane is the key of register r) and
            // its sum (of the rounded values, the ones the second product sees)
            ex4 pb;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pb[r] = (E)__builtin_amdgcn_exp2f(lg[r] - m_ref);
                l_run += (float)pb[r];
            }
            // O^T += V^T P^T: fragments of PV_GROUP value tiles requested together, one group ahead
            ex4 vf[2][PV_GROUP];
            auto request = [&](int grp, int bsel) {
#pragma unroll
                for (int i = 0; i < PV_GROUP; ++i) vf[bsel][i] = lds_read_tr16((lds_b64_ptr)(buf + v_off + 32 * (grp * PV_GROUP + i)));
            };
            request(0, 0);
#pragma unroll
            for (int grp = 0; grp < NDT / PV_GROUP; ++grp) {
                __builtin_amdgcn_sched_barrier(0);
                if (grp + 1 < NDT / PV_GROUP) request(grp + 1, (grp + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < PV_GROUP; ++i) acc[grp * PV_GROUP + i] = mfma_16x16x16(vf[grp & 1][i], pb, acc[grp * PV_GROUP + i]);
            }
        });

        l_tot = l_run + __shfl_xor(l_run, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        if (again || __builtin_amdgcn_ballot_w64(!(l_tot <= SUM_LIMIT)) == 0) break;
        // (wave-uniform) a head ran out of exponent headroom: exact maxima of the range, then the pass again
        m_seen = NEG_BIG;
        sweep([&](int tl, const char *buf) {
            float lg[4];
            tile_logits(tl, buf, lg);
            m_seen = fmaxf(m_seen, head_max(lg));
        });
        again = true;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                      // the last tile's reads are done before the buffers are reused
    char *buf = buf0;                                                       // the merge uses the wavefront's two buffers as one

    // The four wavefronts' results (reference, sum, unnormalised output per head) are merged here, through LDS, so that
    // one partial result per workgroup goes to memory: each wavefront publishes its references and sums, rescales its
    // accumulators to the common reference into its own (now idle) tile buffer, and then adds up a quarter of the
    // value columns over the four buffers.
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
        float *mine = reinterpret_cast<float *>(buf) + col * MROW + 4 * q4;   // [head][MROW] floats, 33 KB of the two buffers' 36.5 KB
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
    // wavefront w adds up value columns [128 w, 128 w + 128) of every head and writes them: as this workgroup's partial
    // result (natural-log units), or -- when the workgroup has the whole (sequence, set) to itself -- normalised, as the
    // final output
    float *dst0 = kp.part + ((size_t)bs * wg_per_bs + blockIdx.x % wg_per_bs) * kp.hps * (DP + 2);
    for (int h = 0; h < kp.hps; ++h) {
        const int x = 128 * wave + 2 * lane;
        float2 sum = float2{0.f, 0.f};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float2 v = *reinterpret_cast<const float2 *>(reinterpret_cast<const float *>(bufs[w][0]) + h * MROW + x);
            sum.x += v.x;
            sum.y += v.y;
        }
        if (kp.O != nullptr) {
            typedef E ex2 __attribute__((ext_vector_type(2)));
            const float inv = 1.f / l_heads[h];
            *reinterpret_cast<ex2 *>(reinterpret_cast<E *>(kp.O) + ((size_t)bs * kp.hps + h) * DP + x) = ex2{(E)(sum.x * inv), (E)(sum.y * inv)};
        } else {
            *reinterpret_cast<float2 *>(dst0 + (size_t)h * (DP + 2) + 2 + x) = sum;
        }
    }
    if (kp.O != nullptr) return;
    if (wave == 0 && q4 == 0 && col < kp.hps) {
        float *dst = dst0 + (size_t)col * (DP + 2);
        dst[0] = m_all == -INFINITY ? -INFINITY : m_all * LN2;
        dst[1] = l_all;
    }
}

}  // namespace

bool decode_mla_supported(const Dims &d)
{
    const int hps = d.H / d.S;
    return (d.dtype == LCA_BF16 || d.dtype == LCA_F16) && d.mode == LCA_MODE_MLA && d.d_pool == DP && d.d_sel == DS && hps <= 16 && d.scale > 0.f;
}

// partial results per (sequence, set): a multiple of 4 (one per wavefront), enough workgroups to fill the chip,
// at least four tiles per wavefront where the cache is long enough
int decode_mla_parts(const Dims &d)
{
    const int tiles = (d.m + BN - 1) / BN + (d.k + BN - 1) / BN;      // (an upper bound when the two kinds share tiles)
    int wgs = (256 + d.B * d.S - 1) / (d.B * d.S);
    const int max_wgs = (tiles + 15) / 16;
    if (wgs > max_wgs) wgs = max_wgs;
    if (wgs < 1) wgs = 1;
    return 4 * wgs;
}

hipError_t launch_decode_mla(const DecodeArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    DmParams kp;
    kp.q = (const uint16_t *)a.q; kp.pool_rep = (const uint16_t *)a.pool_rep; kp.sel_rep = (const uint16_t *)a.sel_rep;
    kp.pool_tail = (const uint16_t *)a.pool_tail; kp.sel_tail = (const uint16_t *)a.sel_tail; kp.part = a.part;
    kp.S = d.S; kp.hps = d.H / d.S; kp.m = d.m; kp.k = d.k; kp.n_parts = a.splits;
    kp.m_cap = a.m_cap; kp.k_cap = a.k_cap; kp.k_start = a.k_start;
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    kp.pool_q8 = a.pool_q8; kp.sel_q8 = a.sel_q8; kp.scales = a.scales;
    kp.O = a.splits == 4 ? a.O : nullptr;
    const unsigned grid = d.B * d.S * (a.splits / 4);
    if (a.pool_q8 != nullptr) {
        if (d.dtype == LCA_F16) decode_mla_kernel<_Float16, true><<<grid, 256, 0, st>>>(kp);
        else decode_mla_kernel<__bf16, true><<<grid, 256, 0, st>>>(kp);
    } else {
        if (d.dtype == LCA_F16) decode_mla_kernel<_Float16, false><<<grid, 256, 0, st>>>(kp);
        else decode_mla_kernel<__bf16, false><<<grid, 256, 0, st>>>(kp);
    }
    return hipGetLastError();
}

}  // namespace lca
