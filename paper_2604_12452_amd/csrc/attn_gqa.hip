// bf16 MFMA attention kernel for the GQA widths (d_k = d_v = 128) on gfx950: prefill over the condensed
// context with hard-selected keys and pooled values per KV head (section 5.4 of the paper; attention as in
// section 4.3, Eq. 10 with the per-query partition of appendix A.2) and, with dense = 1, plain causal
// attention (section 3, Eq. 5).
//
// At d = 128 a (query, key) pair costs 512 MFMA flops and one exponential, so the vector ALU is as busy as
// the matrix core; the kernel therefore keeps its register footprint small enough for two workgroups per
// CU and lets the hardware overlap one wavefront's softmax with another's MFMAs.
//
// Workgroup = 4 wavefronts; a wavefront owns 32 query rows of ONE query head, and the wavefronts of a
// workgroup are the query heads of one KV head (4 heads x 32 rows at 4 heads per KV head), so they share
// every key/value tile and see exactly the same keys.  Tiles of 64 entries (K and V rows of 256 B) are
// copied by direct-to-LDS loads into two 32 KB stages, one tile ahead.  Rows sit at a 256-byte stride with
// their 16-byte chunks XOR-swizzled by row, which keeps both read patterns bank-conflict-free:
//   S^T[key, query] = K Q^T      16-byte key reads, lane = S^T row m reads LDS row pi(m)
//   O^T[dv, query] += V^T P^T    transpose reads (ds_read_b64_tr_b16), each 16-lane block touches rows 4 apart
// with pi(8h + 4G + j) = 4j + 2h + G inside each 16 rows (the S^T accumulator registers then already are
// the B fragments of the second product).  Softmax uses one fixed reference per row (first tile) and a
// repeat pass if the exponent headroom of 2^60 is ever exceeded, so O^T is never rescaled.
#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;                  // d_k = d_v
constexpr int BN = 64;                  // entries per tile (two halves of 32)
constexpr int RB = D * 2;               // row bytes
constexpr int V_OFF = BN * RB;          // the value rows of a stage start here
constexpr int STAGE_BYTES = 2 * BN * RB;   // 32 768
constexpr int NKS = D / 16;             // 8 k-steps of S^T
constexpr int NDV = D / 32;             // 4 value tiles
constexpr int COPIES_PER_TILE = 8;      // direct-to-LDS loads per wavefront and tile (4 for K, 4 for V)
constexpr float NEG_BIG = -1.0e30f;
constexpr float HEADROOM = 60.0f;

struct GqaParams {
    const uint16_t *Q, *K, *V, *k_rep, *v_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, g, w, m, dense;
    int hw, rbs;        // query heads per workgroup (min(H/S, 4)), 32-row blocks per workgroup (4 / hw)
    int n_qb, n_units;  // query blocks per sequence; KV-sharing units = B * S * (H/S / hw)
    float scale_log2, bias_log2;
};

__device__ __forceinline__ int lds_row_of_m(int m) { return (m & 16) + 4 * (m & 3) + 2 * ((m >> 3) & 1) + ((m >> 2) & 1); }
__device__ __forceinline__ int acc_entry(int r, int G) { return lds_row_of_m(8 * (r >> 2) + 4 * G + (r & 3)); }

// One direct-to-LDS load of 64 x 16 bytes (lane l: global [base + voff, +16) -> LDS [lds_addr + 16 l, +16)).
// Inline assembly so that the compiler does not make later LDS reads wait for it; ordering is by hand
// (s_waitcnt vmcnt(0) + workgroup barrier before a stage is read).
__device__ __forceinline__ void dma_1k(unsigned voff, const void *base, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_addr));
}
__device__ __forceinline__ unsigned lds_address(const char *p) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p; }

__global__ __launch_bounds__(256, 2) void attn_gqa_kernel(const GqaParams kp)
{
    __shared__ __attribute__((aligned(1024))) char stages[2][STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, G = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = kp.L, H = kp.H, g = kp.g, w = kp.w;

    // workgroup -> (unit = sequence x KV head x head group, query block); a unit keeps to one XCD when the
    // number of units is a multiple of 8; heaviest (latest) query blocks first
    const int unit = blockIdx.x % kp.n_units, qb = kp.n_qb - 1 - blockIdx.x / kp.n_units;
    const int hps = H / kp.S, hgs = hps / kp.hw;
    const int hg = unit % hgs, s = (unit / hgs) % kp.S, b = unit / (hgs * kp.S);
    const int h = s * hps + hg * kp.hw + wave % kp.hw;      // this wavefront's query head
    const int rb = wave / kp.hw;                             // ... and 32-row block inside the workgroup's rows
    const int BMI = 32 * kp.rbs;

    const int t0 = qb * BMI;
    const int t_last = min(t0 + BMI, L) - 1;
    const int t_wfirst = t0 + rb * 32, t_wlast = t_wfirst + 31;
    const int t_row = t_wfirst + n;
    auto groups_visible = [&](int t) { return (kp.dense || t + 1 <= w) ? 0 : (t + 1 - w) / g; };
    const int mt_row = groups_visible(t_row), raw_lo_row = mt_row * g;
    const int mt_blk_hi = groups_visible(t_last), raw_lo_blk = groups_visible(t0) * g;
    const int mt_w_lo = groups_visible(t_wfirst), mt_w_hi = groups_visible(t_wlast);
    const int n_rep_tiles = (mt_blk_hi + BN - 1) / BN;
    const int n_tiles = n_rep_tiles + (t_last + 1 - raw_lo_blk + BN - 1) / BN;

    // segments: representatives [B,S,m,128] (row stride 256 B), raw tokens [B,L,S,128] (row stride S*256 B)
    const uint16_t *k_rep = kp.k_rep + ((size_t)b * kp.S + s) * kp.m * D, *v_rep = kp.v_rep + ((size_t)b * kp.S + s) * kp.m * D;
    const uint16_t *k_raw = kp.K + ((size_t)b * L * kp.S + s) * D, *v_raw = kp.V + ((size_t)b * L * kp.S + s) * D;
    const int raw_stride = kp.S * RB;

    // copy of tile tl: this wavefront moves rows 16*wave .. 16*wave+15 of K and of V, 4 rows per load; lane l
    // fills slot l&15 of local row l>>4 with the chunk the swizzle assigns to that slot
    const int c0 = (lane & 15) ^ (lane >> 4);
    auto issue_copy = [&](int tl) {
        const bool is_rep = tl < n_rep_tiles;
        const int e0 = is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        const int last = (is_rep ? mt_blk_hi : t_last + 1) - 1;
        const int stride = is_rep ? RB : raw_stride;
        const uint16_t *kb = is_rep ? k_rep : k_raw, *vb = is_rep ? v_rep : v_raw;
        const unsigned st = lds_address(stages[tl & 1]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = 16 * wave + 4 * q;                                   // first of the 4 rows of this load
            const int e = min(e0 + row + (lane >> 4), last);                     // rows past the segment: clamped, masked later
            const unsigned voff = (unsigned)e * stride + ((c0 ^ (4 * q)) << 4);
            dma_1k(voff, kb, st + row * RB);
            dma_1k(voff, vb, st + V_OFF + row * RB);
        }
    };

    // per-lane LDS byte offsets
    const int krow = lds_row_of_m(n), xk = krow & 15;
    int k_off[NKS];                                            // S^T operand: chunk 2ks+G of row krow sits at slot (2ks+G)^xk
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_off[ks] = krow * RB + (((2 * ks + G) ^ xk) << 4);
    int v_off[NDV][2];                                         // V^T operand, per value tile and run h of four keys
    {
        const int p = lane & 15, j = p >> 2, blk = (lane >> 4) & 1, pp = (p & 3) >> 1;
#pragma unroll
        for (int dvt = 0; dvt < NDV; ++dvt)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int row = 4 * j + 2 * hh + G;            // + 16*kk + 32*half
                const int chunk = 4 * dvt + 2 * blk + pp;
                v_off[dvt][hh] = V_OFF + row * RB + ((chunk ^ (row & 15)) << 4) + 8 * (p & 1);
            }
    }

    // Q^T fragments
    bf16x8 qf[NKS];
    {
        const uint16_t *qp = kp.Q + (((size_t)b * L + min(t_row, L - 1)) * H + h) * D + G * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }

    floatx16 acc[NDV];
    float m_ref, l_run, m_seen, m_init = NEG_BIG;
    bool exceeded;
    const float c = kp.scale_log2;
    typedef __attribute__((address_space(3))) bf16x4 *lds_b64_ptr;

restart:
#pragma unroll
    for (int i = 0; i < NDV; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    m_ref = m_init; l_run = 0.f; m_seen = NEG_BIG; exceeded = false;
    issue_copy(0);

    for (int tl = 0; tl < n_tiles; ++tl) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's share of tile tl has landed
        __syncthreads();                                   // ... and everyone's; everyone is done with tile tl-1
        if (tl + 1 < n_tiles) issue_copy(tl + 1);
        const char *cur = stages[tl & 1];
        const bool is_rep = tl < n_rep_tiles;
        const int e_tile = is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        const float bias = is_rep ? kp.bias_log2 : 0.f;

#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const int e0 = e_tile + half * 32;
            const bool none = is_rep ? (e0 >= mt_w_hi) : (e0 > t_wlast || e0 + 32 <= mt_w_lo * g);
            if (none) continue;                            // no row of this wavefront sees this half (wave-uniform)
            const bool full = is_rep ? (e0 + 32 <= mt_w_lo) : (e0 + 31 <= t_wfirst && e0 >= mt_w_hi * g);
            const char *hb = cur + half * 32 * RB;

            // S^T = K Q^T
            floatx16 sacc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(hb + k_off[ks]);
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
            }
            // mask, maximum, reference
            if (!full) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int e = e0 + acc_entry(r, G);
                    const bool vis = is_rep ? (e < mt_row) : (e >= raw_lo_row && e <= t_row);
                    sacc[r] = vis ? sacc[r] : -INFINITY;
                }
            }
            float tmax = sacc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sacc[r]);
            tmax = fmaxf(fmaf(tmax, c, bias), NEG_BIG);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            m_ref = (m_ref == NEG_BIG) ? tmax : m_ref;     // first visible keys of this row fix its reference
            m_seen = fmaxf(m_seen, tmax);
            exceeded |= tmax > m_ref + HEADROOM;
            const float nb = bias - m_ref;
            // P^T = exp2(S^T * c + bias - ref): registers 0..7 / 8..15 are the two k-steps of the second product
            bf16x8 pb[2];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[kk * 8 + i], c, nb));
                    l_run += pv;
                    pb[kk][i] = (__bf16)pv;
                }
            // O^T += V^T P^T
#pragma unroll
            for (int dvt = 0; dvt < NDV; ++dvt)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const char *vb = hb + kk * 16 * RB;
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vb + v_off[dvt][0]));
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vb + v_off[dvt][1]));
                    const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    acc[dvt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kk], acc[dvt], 0, 0, 0);
                }
        }
    }

    // every wavefront is done with the stages; repeat the pass if any row ran out of exponent headroom
    if (__syncthreads_or(exceeded)) {
        m_init = m_seen;
        goto restart;
    }

    // epilogue: normalise, transpose through LDS, store rows of 256 B coalesced
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.f / l_tot;
    constexpr int ORS = RB + 16;
    static_assert(4 * 32 * ORS <= 2 * STAGE_BYTES, "output staging must fit in the stages");
    char *obuf = &stages[0][0] + wave * 32 * ORS;
#pragma unroll
    for (int dvt = 0; dvt < NDV; ++dvt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            union { bf16x4 h; uint2 u; } o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)(acc[dvt][r4 * 4 + i] * inv);
            *reinterpret_cast<uint2 *>(obuf + n * ORS + (dvt * 32 + 8 * r4 + 4 * G) * 2) = o.u;
        }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int r4 = 0; r4 < 8; ++r4) {                         // one wave-wide store covers four rows
        const int r = r4 * 4 + (lane >> 4), t = t_wfirst + r;
        const uint4 v = *reinterpret_cast<const uint4 *>(obuf + r * ORS + (lane & 15) * 16);
        if (t < L) *reinterpret_cast<uint4 *>(kp.O + (((size_t)b * L + t) * H + h) * D + (lane & 15) * 8) = v;
    }
    if (kp.lse != nullptr && G == 0 && t_row < L) kp.lse[((size_t)b * L + t_row) * H + h] = (m_ref + log2f(l_tot)) * 0.6931471805599453f;
}

}  // namespace

bool attn_gqa_supported(const Dims &d)
{
    const int hps = d.H / d.S;
    return d.dtype == LCA_BF16 && d.mode == LCA_MODE_GQA && d.d_pool == D && d.d_sel == D && d.scale > 0.f &&
           (hps == 1 || hps == 2 || hps % 4 == 0) && (long)d.L * d.S * RB < (1l << 31);
}

hipError_t launch_attn_gqa(const AttnArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    GqaParams kp;
    kp.Q = (const uint16_t *)a.Q; kp.K = (const uint16_t *)a.SEL; kp.V = (const uint16_t *)a.POOL;
    kp.k_rep = (const uint16_t *)a.sel_rep; kp.v_rep = (const uint16_t *)a.pool_rep;
    kp.O = (uint16_t *)a.O; kp.lse = a.lse;
    kp.B = d.B; kp.L = d.L; kp.H = d.H; kp.S = d.S; kp.g = d.g; kp.w = d.w; kp.m = d.m; kp.dense = a.dense;
    const int hps = d.H / d.S;
    kp.hw = hps < 4 ? hps : 4;
    kp.rbs = 4 / kp.hw;
    kp.n_qb = (d.L + 32 * kp.rbs - 1) / (32 * kp.rbs);
    kp.n_units = d.B * d.S * (hps / kp.hw);
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    const long grid = (long)kp.n_units * kp.n_qb;
    attn_gqa_kernel<<<(unsigned)grid, 256, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
