// bf16 MFMA attention kernel for gfx950: prefill over the condensed context (section 4.3, Eq. 10;
// per-query partition of appendix A.2) and, with dense = 1, plain causal attention (section 3, Eq. 5).
//
// Work split: one workgroup (4 wavefronts) per (sequence, head, block of 128 query rows); each
// wavefront owns 32 query rows and the whole value width.  Key tiles of 32 entries go through LDS
// once and are used twice: as the key (all columns of the row in MLA mode) and as the value (the
// first d_pool columns) — the absorbed MLA form needs no separate value tile.
//
// The product is computed transposed so that no data has to change lanes between the two MFMA
// stages:   S^T[key, query] = K Q^T      (A = key tile from LDS, B = Q^T held in registers)
//           O^T[dv,  query] += V^T P^T   (A = V^T from LDS,      B = P^T = exp2(S^T - max), bf16)
// In the 32x32 accumulator layout lane l holds query column l%32, so the softmax statistics are one
// scalar per lane, and the S^T accumulator registers already are B-operand fragments for the second
// product once the keys of the V^T operand are read in the matching order.
#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 32;    // entries per key tile
constexpr int PAD = 8;    // LDS row padding (elements) — keeps 16-byte row reads conflict-free

struct KParams {
    const uint16_t *Q, *POOL, *SEL, *pool_rep, *sel_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, P, g, w, m, dense, n_qb;
    float scale_log2, bias_log2;
};

// key row held in accumulator register r of lane group G (lanes 32G..32G+31) of a 32x32 tile
__device__ __forceinline__ int acc_row(int r, int G) { return 8 * (r >> 2) + 4 * G + (r & 3); }

template <int DP, int DS, bool MLA>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const KParams kp)
{
    constexpr int DQK = MLA ? DP + DS : DS;
    constexpr int DV = DP;
    constexpr int ROWW = DP + DS;            // tile row = [pool | sel]
    constexpr int RS = ROWW + PAD;           // LDS row stride in elements
    constexpr int KOFF = MLA ? 0 : DP;       // first key column inside the tile row
    constexpr int NKS = DQK / 16;            // k-steps of S^T
    constexpr int NDV = DV / 32;             // 32-wide value tiles
    constexpr int NCP = DP / 8, CPR = ROWW / 8;   // 16-byte chunks: pool part, whole row
    constexpr int NCHUNK = BN * CPR;
    static_assert(DQK % 16 == 0 && DV % 32 == 0, "shape");

    __shared__ __attribute__((aligned(16))) uint16_t tile[BN * RS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, G = lane >> 5;

    // Workgroup -> (sequence, head, query block).  Consecutive workgroup ids go to different XCDs, so
    // ids with equal id%8 walk the heads of one query block back to back on one XCD (shared K/V stays
    // in that XCD's L2), and blocks are issued heaviest (latest rows) first.
    const int xcd = blockIdx.x & 7, kidx = blockIdx.x >> 3;
    const int h = kidx % kp.H;
    const int ord = (kidx / kp.H) * 8 + xcd;
    if (ord >= kp.n_qb * kp.B) return;
    const int b = ord % kp.B;
    const int qb = kp.n_qb - 1 - ord / kp.B;
    const int L = kp.L, H = kp.H, g = kp.g, w = kp.w;
    const int s = h / (H / kp.S), p = MLA ? 0 : s, P = kp.P;

    const int t0 = qb * BM;
    const int t_last = min(t0 + BM, L) - 1;
    const int t_row = t0 + wave * 32 + n;                 // this lane's query row
    const int t_wfirst = t0 + wave * 32, t_wlast = t0 + wave * 32 + 31;

    auto groups_visible = [&](int t) { return (kp.dense || t + 1 <= w) ? 0 : (t + 1 - w) / g; };
    const int mt_row = groups_visible(t_row), raw_lo_row = mt_row * g;
    const int mt_blk_lo = groups_visible(t0), mt_blk_hi = groups_visible(t_last);
    const int mt_w_lo = groups_visible(t_wfirst), mt_w_hi = groups_visible(t_wlast);
    const int raw_lo_blk = mt_blk_lo * g;
    const int n_rep_tiles = (mt_blk_hi + BN - 1) / BN;
    const int n_raw_tiles = (t_last + 1 - raw_lo_blk + BN - 1) / BN;

    // Q^T fragments: lane (n, G) holds Q[t_row, ks*16 + 8G .. +7]
    bf16x8 qf[NKS];
    {
        const uint16_t *qp = kp.Q + (((size_t)b * L + min(t_row, L - 1)) * H + h) * DQK + G * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }

    floatx16 acc[NDV];
#pragma unroll
    for (int i = 0; i < NDV; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const uint16_t *rep_pool = kp.pool_rep + ((size_t)b * kp.S + s) * kp.m * DP;
    const uint16_t *rep_sel = kp.sel_rep + ((size_t)b * kp.S + s) * kp.m * DS;
    const uint16_t *raw_pool = kp.POOL + ((size_t)b * L * P + p) * DP;
    const uint16_t *raw_sel = kp.SEL + ((size_t)b * L * P + p) * DS;

    for (int tl = 0; tl < n_rep_tiles + n_raw_tiles; ++tl) {
        const bool is_rep = tl < n_rep_tiles;
        const int e0 = is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        const int seg_end = is_rep ? mt_blk_hi : t_last + 1;
        const uint16_t *pbase = is_rep ? rep_pool : raw_pool;
        const uint16_t *sbase = is_rep ? rep_sel : raw_sel;
        const size_t pstride = is_rep ? DP : (size_t)P * DP, sstride = is_rep ? DS : (size_t)P * DS;

        __syncthreads();   // everyone is done with the previous tile
        for (int q = tid; q < NCHUNK; q += 256) {
            const int r = q / CPR, c = q % CPR;
            const int e = min(e0 + r, seg_end - 1);        // clamp: rows past the segment are masked below
            const uint16_t *src = c < NCP ? pbase + (size_t)e * pstride + c * 8 : sbase + (size_t)e * sstride + (c - NCP) * 8;
            *reinterpret_cast<uint4 *>(&tile[r * RS + c * 8]) = *reinterpret_cast<const uint4 *>(src);
        }
        __syncthreads();

        // skip tiles no row of this wavefront can see (wave-uniform)
        const bool none = is_rep ? (e0 >= mt_w_hi) : (e0 > t_wlast || e0 + BN <= mt_w_lo * g);
        if (none) continue;
        const bool full = is_rep ? (e0 + BN <= mt_w_lo) : (e0 + BN - 1 <= t_wfirst && e0 >= mt_w_hi * g);

        // S^T = K Q^T
        floatx16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&tile[n * RS + KOFF + ks * 16 + G * 8]);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
        }

        // scaled logits (base 2), mask, running maximum
        const float bias = is_rep ? kp.bias_log2 : 0.f;
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = fmaf(sacc[r], kp.scale_log2, bias);
            if (!full) {
                const int e = e0 + acc_row(r, G);
                const bool vis = is_rep ? (e < mt_row) : (e >= raw_lo_row && e <= t_row);
                v = vis ? v : -INFINITY;
            }
            sacc[r] = v;
            tmax = fmaxf(tmax, v);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);
        const float m_eff = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_eff);
        float lsum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            sacc[r] = exp2f(sacc[r] - m_eff);
            lsum += sacc[r];
        }
        l_run = l_run * alpha + lsum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < NDV; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] *= alpha;

        // P^T fragments: registers 0..7 and 8..15 are the two k-steps of the second product
        bf16x8 pb[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 8; ++i) pb[kk][i] = (__bf16)sacc[kk * 8 + i];

        // O^T += V^T P^T ; lane (n, G) supplies V[key(kk, G, i)][dvt*32 + n], keys in accumulator order
#pragma unroll
        for (int dvt = 0; dvt < NDV; ++dvt) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                union { bf16x8 v; uint16_t u[8]; } a;
#pragma unroll
                for (int i = 0; i < 8; ++i) a.u[i] = tile[(kk * 16 + acc_row(i, G)) * RS + dvt * 32 + n];
                acc[dvt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pb[kk], acc[dvt], 0, 0, 0);
            }
        }
    }

    // epilogue: normalise and store. Lane (n, G) holds, for query row t_row, value columns
    // dvt*32 + 8*(r/4) + 4G + r%4 — four consecutive columns per r/4.
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (t_row < L) {
        const float inv = 1.f / l_tot;
        uint16_t *op = kp.O + (((size_t)b * L + t_row) * H + h) * DV;
#pragma unroll
        for (int dvt = 0; dvt < NDV; ++dvt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)(acc[dvt][r4 * 4 + i] * inv);
                *reinterpret_cast<uint2 *>(op + dvt * 32 + 8 * r4 + 4 * G) = o.u;
            }
        if (kp.lse != nullptr && G == 0)
            kp.lse[((size_t)b * L + t_row) * H + h] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
}

template <int DP, int DS, bool MLA>
hipError_t run(const AttnArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    KParams kp;
    kp.Q = (const uint16_t *)a.Q; kp.POOL = (const uint16_t *)a.POOL; kp.SEL = (const uint16_t *)a.SEL;
    kp.pool_rep = (const uint16_t *)a.pool_rep; kp.sel_rep = (const uint16_t *)a.sel_rep;
    kp.O = (uint16_t *)a.O; kp.lse = a.lse;
    kp.B = d.B; kp.L = d.L; kp.H = d.H; kp.S = d.S; kp.P = d.P; kp.g = d.g; kp.w = d.w; kp.m = d.m; kp.dense = a.dense;
    kp.n_qb = (d.L + BM - 1) / BM;
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    const long units = (long)kp.n_qb * d.B;
    const long grid = ((units + 7) / 8) * 8 * d.H;
    attn_mfma_kernel<DP, DS, MLA><<<(unsigned)grid, 256, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(const Dims &d)
{
    if (d.dtype != LCA_BF16) return false;
    if (d.mode == LCA_MODE_MLA) return d.d_pool == 512 && d.d_sel == 64;
    return d.d_pool == 128 && d.d_sel == 128;
}

hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t st)
{
    if (a.d.mode == LCA_MODE_MLA) return run<512, 64, true>(a, st);
    return run<128, 128, false>(a, st);
}

}  // namespace lca
