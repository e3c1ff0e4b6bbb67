// Latent-space condensation at the MLA widths (d_c = 512, d_R = 64, bf16 or fp16) with several condensed sets, on the
// matrix cores (section 4.2 of the paper; Algorithm 1, loop over groups; Eq. 6-8).
//
// With S condensed sets the g rows of a group meet S summary queries: scores are a (g x 576)(576 x S) product and the pooled
// vectors a (512 x g)(g x S) product.  On the vector ALU that is 2 S (576 + 512) multiply-adds per row of 1152 bytes -- 30
// flops per byte at S = 16, beyond what the vector ALU does at HBM speed -- so both products run as 16x16 MFMAs with the sets
// as the 16 columns, on tiles of 16 rows copied straight into LDS:
//   S^T[row, set]   = K Qbar^T      A = 16 key rows from LDS (16-byte reads), B = summary queries in registers (18 k-steps)
//   C^T[dv, set]   += V^T P^T       A = V^T through LDS transpose reads,       B = P^T = exp2(S^T - max)
// Precision: the inputs are 16-bit, products are exact and sums are fp32 inside the matrix core; the two fp32 operands of the
// method -- the summary query and the softmax weights -- enter as the sum of two 16-bit numbers (value = hi + lo, each product
// done twice), which keeps 16 (bf16) or 22 (fp16) of their mantissa bits: scores and pooled vectors are fp32-accurate to
// about 1e-5 relative, far inside the score margin below which anchors may differ from a float64 evaluation.  A summary
// query is first scaled by a power of two so that its largest component lies in [1, 2) (fp16's narrow exponent range).
// Equal rows of a group get equal score bits (every row of a tile goes through the same sequence of operations), so exact
// ties go to the lowest index.
//
// Persistent kernel, one workgroup per CU, every WAVEFRONT works alone on its own groups with two 18 KB tile buffers: the
// copy of the next tile travels while the current one is used; there is no barrier anywhere.  With one wavefront per SIMD
// every instruction costs its full issue latency, so the summary queries themselves (Algorithm 1, step 1) stay in the small
// kernel launched in front of this one: computed here, once per workgroup, they took longer than that launch.
#include "lca_internal.h"
#include "mla_tile16.h"

namespace lca {
namespace {

using namespace tile16;

constexpr int NKS = DQK / 32;                   // 18 k-steps of S^T
constexpr int NDT = DP / 16;                    // 32 value tiles
constexpr int PV_GROUP = 4;                     // value tiles whose V^T fragments are requested together
constexpr int WAVES = 4;
constexpr unsigned BSTRIDE = WAVES * BUF_BYTES; // a wavefront's two tile buffers are this far apart
constexpr float LOG2E = 1.4426950408889634f;

struct CmParams {
    const uint16_t *POOL, *SEL;
    uint16_t *pool_rep, *sel_rep;
    int32_t *anchor;
    float *alpha_dbg;
    const float *qbar;                     // summary queries [B, S, 576] (summary_query_kernel)
    int B, L, S, m, G;
    float scale;
};

template <typename E>
__global__ __launch_bounds__(256, 1) void condense_mfma_kernel(const CmParams kp)
{
    typedef E ex8 __attribute__((ext_vector_type(8)));
    typedef E ex4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) ex4 *lds_b64_ptr;
    __shared__ __attribute__((aligned(1024))) char bufs[2][WAVES][BUF_BYTES];   // [buffer][wavefront]

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 15, q4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_waves = gridDim.x * WAVES, wave_gid = blockIdx.x * WAVES + wave;
    const int S = kp.S, m = kp.m, G = kp.G, tpg = G / BN;
    if ((int)blockIdx.x * WAVES >= m) return;               // (the grid is sized so that this never happens)
    const int my_groups = wave_gid < m ? (m - wave_gid + n_waves - 1) / n_waves : 0;
    const int my_tiles = my_groups * tpg;
    char *buf0 = bufs[0][wave];
    const unsigned buf_lds = lds_address(buf0);

    // per-lane LDS offsets inside a tile buffer (the layout and the row permutation of the decode kernel)
    const int krow = 4 * (col & 3) + (col >> 2);            // LDS row behind S^T row `col` of the tile's 16 rows
    const int k_off = krow * RSB + 16 * q4;                 // + 64*ks
    const int ksel_row = SEL_OFF + krow * (DS * 2);         // chunk c at slot c ^ (row & 7)
    const int v_off = (4 * (col >> 2) + q4) * RSB + 8 * (col & 3);   // + 32*t: transpose read of 4 rows (4 apart) x 4 columns

    for (int b = 0; b < kp.B; ++b) {
        const uint16_t *pool_b = kp.POOL + (size_t)b * kp.L * DP, *sel_b = kp.SEL + (size_t)b * kp.L * DS;
        // tile n of this wavefront: rows [row0, row0 + 16) of the sequence
        auto tile_row0 = [&](int n) { return (wave_gid + (n / tpg) * n_waves) * G + (n % tpg) * BN; };
        auto issue_dma = [&](int n, int bi) {
            const int row0 = tile_row0(n);
            const unsigned dst = buf_lds + bi * BSTRIDE;
            const char *pb0 = (const char *)(pool_b + (size_t)row0 * DP), *sb0 = (const char *)(sel_b + (size_t)row0 * DS);
#pragma unroll
            for (int r = 0; r < BN; ++r) dma_row(lane * 16, pb0 + r * (DP * 2), dst + r * RSB);
#pragma unroll
            for (int j = 0; j < BN / 8; ++j) {
                const int r = 8 * j + (lane >> 3);
                dma_row(r * (DS * 2) + (((lane & 7) ^ (r & 7)) << 4), sb0, dst + SEL_OFF + 8 * j * (DS * 2));
            }
        };

        // ---- this lane's B fragments of the summary queries of sequence b (Algorithm 1, step 1: computed by the kernel launched
        // before this one), while the first tile travels: set `col`, components 32 ks + 8 q4 .. +7, as hi + lo of the query scaled
        // by a power of two ----
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // this wavefront's reads of the previous sequence's last tile are done
        if (my_tiles > 0) issue_dma(0, 0);
        ex8 qhi[NKS], qlo[NKS];
        float c2;                                               // base-2 logit = accumulator * c2
        {
            const float *src = kp.qbar + ((size_t)b * S + min(col, S - 1)) * DQK + 8 * q4;
            floatx4 qa[NKS], qb[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                qa[ks] = *reinterpret_cast<const floatx4 *>(src + 32 * ks);
                qb[ks] = *reinterpret_cast<const floatx4 *>(src + 32 * ks + 4);
            }
            float mx = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int e = 0; e < 4; ++e) mx = fmaxf(mx, fmaxf(fabsf(qa[ks][e]), fabsf(qb[ks][e])));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            // pre = 2^-floor(log2 mx) (1 for a zero query), built from the exponent bits; exact, and so is its reciprocal
            const int biased = (int)((__float_as_uint(mx) >> 23) & 255u);
            const int pre_exp = mx == 0.f ? 127 : min(254, max(1, 254 - biased));
            const float pre = __uint_as_float((unsigned)pre_exp << 23), inv_pre = __uint_as_float((unsigned)(254 - pre_exp) << 23);
            c2 = kp.scale * LOG2E * inv_pre;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = col < S ? (e < 4 ? qa[ks][e] : qb[ks][e - 4]) * pre : 0.f;
                    const E hi = (E)x;
                    qhi[ks][e] = hi;
                    qlo[ks][e] = (E)(x - (float)hi);
                }
        }

        // ---- loop over this wavefront's tiles ----
        floatx4 acc[NDT];
        float m_run = -INFINITY, l_run = 0.f, best = -INFINITY;
        int best_e = 0;
        bool landed = false;                                    // the copy of the tile about to be used has been waited for
        uint4 sel_best[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
        for (int n = 0; n < my_tiles; ++n) {
            const int bi = n & 1, tt = n % tpg;
            const int j = wave_gid + (n / tpg) * n_waves;       // group
            char *buf = buf0 + bi * BSTRIDE;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wavefront's reads of tile n-1 (and of its output staging) are done
            if (!landed) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // tile n (a group's last tile waits for its successor itself)
            landed = false;
            if (n + 1 < my_tiles) issue_dma(n + 1, bi ^ 1);
            if (tt == 0) {
#pragma unroll
                for (int t = 0; t < NDT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
                m_run = -INFINITY; l_run = 0.f; best = -INFINITY; best_e = 0;
            }
            // S^T = K Qbar^T (Eq. 6): accumulator register r of this lane is row 4 r + q4 of the tile, for set `col`
            float lg[4];
            {
                constexpr int KC = 6;                           // key fragments per request: chunk i+1 is read while chunk i is multiplied
                ex8 kf[2][KC];
                auto request = [&](int c0, int bsel) {
#pragma unroll
                    for (int i = 0; i < KC; ++i) {
                        const int ks = c0 + i;
                        const char *p = ks < DP / 32 ? buf + k_off + 64 * ks : buf + ksel_row + (((4 * (ks - DP / 32) + q4) ^ (krow & 7)) << 4);
                        kf[bsel][i] = *reinterpret_cast<const ex8 *>(p);
                    }
                };
                request(0, 0);
                floatx4 s_lo = floatx4{0.f, 0.f, 0.f, 0.f}, s_hi = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ch = 0; ch < NKS / KC; ++ch) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (ch + 1 < NKS / KC) request((ch + 1) * KC, (ch + 1) & 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < KC; ++i) {
                        s_lo = mfma_16x16x32(kf[ch & 1][i], qlo[ch * KC + i], s_lo);
                        s_hi = mfma_16x16x32(kf[ch & 1][i], qhi[ch * KC + i], s_hi);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) lg[r] = (s_hi[r] + s_lo[r]) * c2;
            }
            if (kp.alpha_dbg != nullptr && col < S) {           // scores now, turned into weights when the group is complete
                float *ap = kp.alpha_dbg + (((size_t)b * S + col) * m + j) * G + tt * BN;
#pragma unroll
                for (int r = 0; r < 4; ++r) ap[4 * r + q4] = lg[r];
            }
            // largest score of the tile and its lowest row (Eq. 8); rows of a lane ascend with r, lanes of a set with q4
            float tmax = lg[0];
            int te = q4;
#pragma unroll
            for (int r = 1; r < 4; ++r)
                if (lg[r] > tmax) { tmax = lg[r]; te = 4 * r + q4; }
#pragma unroll
            for (int mask = 16; mask <= 32; mask <<= 1) {
                const float os = __shfl_xor(tmax, mask, 64);
                const int oe = __shfl_xor(te, mask, 64);
                if (os > tmax || (os == tmax && oe < te)) { tmax = os; te = oe; }
            }
            const bool improved = tmax > best;                  // an earlier tile of the group wins ties
            if (improved) { best = tmax; best_e = tt * BN + te; }
            // the RoPE key of the best row so far, kept by the lanes that will write it (8 lanes per set, sets 8 p + lane / 8): taken
            // from the tile in LDS -- a load from memory here would have to wait for the next tile's copy, which is in flight
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                if (p == 1 && S <= 8) break;
                const int src_lane = min(8 * p + (lane >> 3), S - 1);
                const bool imp = __shfl((int)improved, src_lane, 64) != 0;
                const int row = __shfl(te, src_lane, 64);
                if (imp) sel_best[p] = *reinterpret_cast<const uint4 *>(buf + SEL_OFF + row * (DS * 2) + (((lane & 7) ^ (row & 7)) << 4));
            }
            // group softmax, online over the group's tiles (Eq. 6), and the pooled sum (Eq. 7)
            const float m_new = fmaxf(m_run, tmax);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);     // 0 on the group's first tile
            m_run = m_new;
            l_run *= corr;
            if (tt > 0) {
#pragma unroll
                for (int t = 0; t < NDT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[t][r] *= corr;
            }
            ex4 phi, plo;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(lg[r] - m_new);
                l_run += p;
                phi[r] = (E)p;
                plo[r] = (E)(p - (float)phi[r]);
            }
            {
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
                    for (int i = 0; i < PV_GROUP; ++i) {
                        acc[grp * PV_GROUP + i] = mfma_16x16x16(vf[grp & 1][i], plo, acc[grp * PV_GROUP + i]);
                        acc[grp * PV_GROUP + i] = mfma_16x16x16(vf[grp & 1][i], phi, acc[grp * PV_GROUP + i]);
                    }
                }
            }
            if (tt != tpg - 1) continue;

            // ---- the group is complete: representative j of every set ----
            float l_tot = l_run + __shfl_xor(l_run, 16, 64);
            l_tot += __shfl_xor(l_tot, 32, 64);
            const float inv = 1.f / l_tot;
            const int a_tok = j * G + best_e;
            // pooled vectors: accumulator tile t, register r = component 16 t + 4 q4 + r of set `col`; staged in this tile's buffer
            // (all its reads are done) as [set][512] so that every set's row leaves as one contiguous kilobyte
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (col < S) {
#pragma unroll
                for (int t = 0; t < NDT; ++t) {
                    ex4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = (E)(acc[t][r] * inv);
                    *reinterpret_cast<ex4 *>(buf + col * RSB + (16 * t + 4 * q4) * 2) = o;
                }
            }
            // The next tile's copy is waited for HERE, before this group's stores are issued: waited for after them, at the top of
            // the next iteration, the wait would also cover the stores' acknowledgement by memory (loads and stores share one
            // counter).  This way the stores have the whole next tile to complete.
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            landed = true;
            for (int s = 0; s < S; ++s) {
                const uint4 v = *reinterpret_cast<const uint4 *>(buf + s * RSB + 16 * lane);
                *reinterpret_cast<uint4 *>(kp.pool_rep + (((size_t)b * S + s) * m + j) * DP + 8 * lane) = v;
            }
            // anchors and the anchors' RoPE keys, copied bit for bit
            if (q4 == 0 && col < S) kp.anchor[((size_t)b * S + col) * m + j] = a_tok;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int s = 8 * p + (lane >> 3);
                if (s < S) *reinterpret_cast<uint4 *>(kp.sel_rep + (((size_t)b * S + s) * m + j) * DS + 8 * (lane & 7)) = sel_best[p];
            }
            if (kp.alpha_dbg != nullptr && col < S) {           // each lane turns the scores it wrote into weights
                float *ap = kp.alpha_dbg + (((size_t)b * S + col) * m + j) * G;
                for (int t2 = 0; t2 < tpg; ++t2)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float *a1 = ap + t2 * BN + 4 * r + q4;
                        *a1 = __builtin_amdgcn_exp2f(*a1 - m_run) * inv;
                    }
            }
        }
    }
}

}  // namespace

// Descriptors this kernel takes: the MLA widths in a 16-bit type, the method's own reduce strategies, groups that are whole
// tiles of 16 rows, at most 16 sets (the sets are the 16 columns of the products).
bool condense_mla_mfma_supported(const Dims &d)
{
    return (d.dtype == LCA_BF16 || d.dtype == LCA_F16) && d.mode == LCA_MODE_MLA && d.d_pool == DP && d.d_sel == DS && d.S <= 16 &&
           d.g % BN == 0 && d.g <= 64 && d.m > 0 && d.pool_reduce == LCA_REDUCE_WEIGHTED && d.sel_reduce == LCA_REDUCE_MAXSEL &&
           (long)d.L * DP * 2 < (1l << 32);
}

hipError_t launch_condense_mla_mfma(const CondenseArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    CmParams kp;
    kp.POOL = (const uint16_t *)a.POOL; kp.SEL = (const uint16_t *)a.SEL;
    kp.pool_rep = (uint16_t *)a.pool_rep; kp.sel_rep = (uint16_t *)a.sel_rep; kp.anchor = a.anchor; kp.alpha_dbg = a.alpha_dbg;
    kp.B = d.B; kp.L = d.L; kp.S = d.S; kp.m = d.m; kp.G = d.g; kp.scale = d.scale;
    kp.qbar = a.qbar;
    const int wgs_needed = (d.m + WAVES - 1) / WAVES, cus = persistent_grid();
    const unsigned grid = (unsigned)(wgs_needed < cus ? wgs_needed : cus);
    if (d.dtype == LCA_F16) condense_mfma_kernel<_Float16><<<grid, 256, 0, st>>>(kp);
    else condense_mfma_kernel<__bf16><<<grid, 256, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
