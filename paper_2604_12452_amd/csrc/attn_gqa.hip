// bf16 MFMA attention kernel for the GQA widths (d_k = d_v = 128) on gfx950: prefill over the condensed
// context with hard-selected keys and pooled values per KV head (section 5.4 of the paper; attention as in
// section 4.3, Eq. 10 with the per-query partition of appendix A.2) and, with dense = 1, plain causal
// attention (section 3, Eq. 5).
//
// At d = 128 a (query, key) pair costs 512 MFMA flops and one exponential, so the vector ALU is nearly as
// busy as the matrix core; the kernel keeps its register footprint at 256 so that two wavefronts share a
// SIMD, and mixes matrix and vector instructions evenly in program order (see the pass loop).
//
// Workgroup = 8 wavefronts; a wavefront owns 32 query rows of ONE query head, and the wavefronts of a
// workgroup are (the query heads of one KV head) x (blocks of 32 rows): 4 heads x 64 rows at 4 heads per KV
// head, so they share every key/value tile and see exactly the same keys.  Tiles of 64 entries (K and V
// rows of 256 B) are copied by direct-to-LDS loads into four 32 KB stages, two tiles ahead.  Rows sit at a
// 256-byte stride with their 16-byte chunks XOR-swizzled by row (at the source address of the copy), which
// keeps both read patterns bank-conflict-free:
//   S^T[key, query] = K Q^T      16-byte key reads, lane = S^T row m reads LDS row pi(m)
//   O^T[dv, query] += V^T P^T    transpose reads (ds_read_b64_tr_b16), each 16-lane block touches rows 4 apart
// with pi(8h + 4G + j) = 4j + 2h + G inside each 16 rows (the S^T accumulator registers then already are
// the B fragments of the second product).  Softmax uses one fixed reference per row (the first entries the
// row sees), so O^T is never rescaled and no maxima are taken in the steady state; row sums that end beyond
// 2^100 make the workgroup repeat the work from exact maxima.
#include <type_traits>

#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;                  // d_k = d_v
constexpr int BN = 64;                  // entries per tile (two halves of 32)
constexpr int RB = D * 2;               // row bytes
constexpr int V_OFF = BN * RB;          // the value rows of a stage start here
constexpr int STAGE_BYTES = 2 * BN * RB;   // 32 768
constexpr int NSTAGE = 4;               // two pairs of tiles: one in use, one on its way
constexpr int NW = 8;                   // wavefronts per workgroup
constexpr int NKS = D / 16;             // 8 k-steps of S^T
constexpr int NDV = D / 32;             // 4 value tiles
constexpr float NEG_BIG = -1.0e30f;

struct GqaParams {
    const uint16_t *Q, *K, *V, *k_rep, *v_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, g, w, m, dense;
    int hw, rbs;        // query heads per workgroup (min(H/S, 4)), 32-row blocks per workgroup (8 / hw)
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

__global__ __launch_bounds__(64 * NW, 1) void attn_gqa_kernel(const GqaParams kp)
{
    __shared__ __attribute__((aligned(1024))) char stages[NSTAGE][STAGE_BYTES];

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

    // copy of tile tl: this wavefront moves rows 8*wave .. 8*wave+7 of K and of V, 4 rows per load; lane l
    // fills slot l&15 of local row l>>4 with the chunk the swizzle assigns to that slot
    constexpr int RPW = BN / NW, NQ = RPW / 4;                 // rows and loads (per operand) per wavefront
    const int lrow = lane >> 4;
    const int ksw = ((lane & 15) ^ lrow) << 4, vsw = (lane & 15) << 4;   // K: chunk ^ (row & 15); V: chunk ^ (row & 12)
    auto issue_copy = [&](int tl) {
        const bool is_rep = tl < n_rep_tiles;
        const int e0 = (is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN) + RPW * wave;
        const int last = (is_rep ? mt_blk_hi : t_last + 1) - 1;
        const int stride = is_rep ? RB : raw_stride;
        const char *kb = (const char *)(is_rep ? k_rep : k_raw), *vb = (const char *)(is_rep ? v_rep : v_raw);
        const unsigned st = lds_address(stages[tl & (NSTAGE - 1)]) + RPW * wave * RB;
        const bool inside = e0 + RPW - 1 <= last;               // else rows past the segment: clamped, masked later
        const char *kt = kb + (inside ? (size_t)e0 * stride : 0), *vt = vb + (inside ? (size_t)e0 * stride : 0);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int swz = (((RPW * wave) & 8) ^ (4 * q)) << 4;   // bits 2..3 of the row, uniform
            const unsigned rowoff = inside ? (unsigned)(4 * q + lrow) * stride : (unsigned)min(e0 + 4 * q + lrow, last) * stride;
            dma_1k(rowoff + (ksw ^ swz), kt, st + 4 * q * RB);
            dma_1k(rowoff + (vsw ^ swz), vt, st + V_OFF + 4 * q * RB);
        }
    };

    // per-lane LDS addresses of the operand fragments in the current stage (they alternate between the stages
    // as the tiles go by); halves and k-steps are immediate offsets
    const int krow = lds_row_of_m(n), xk = krow & 15;
    const unsigned stage0 = lds_address(stages[0]);
    unsigned k_addr[NKS];                                      // S^T operand: chunk 2ks+G of row krow sits at slot (2ks+G)^xk
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_addr[ks] = stage0 + krow * RB + (((2 * ks + G) ^ xk) << 4);
    unsigned v_addr[NDV];                                      // V^T operand per value tile: chunk c of row r sits at slot c^(r&12)
    {
        const int p = lane & 15, j = p >> 2, blk = (lane >> 4) & 1, pp = (p & 3) >> 1;
#pragma unroll
        for (int dvt = 0; dvt < NDV; ++dvt) {
            const int row = 4 * j + G;                         // + 2*hh + 16*kk + 32*half
            const int chunk = 4 * dvt + 2 * blk + pp;
            v_addr[dvt] = stage0 + V_OFF + row * RB + ((chunk ^ (4 * j)) << 4) + 8 * (p & 1);
        }
    }

    // Q^T fragments
    bf16x8 qf[NKS];
    {
        const uint16_t *qp = kp.Q + (((size_t)b * L + min(t_row, L - 1)) * H + h) * D + G * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
        // the loads complete here: otherwise the compiler waits for them (and with them for every tile copy
        // issued in between) inside the tile loop
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) asm volatile("" : "+v"(qf[ks]));
    }

    floatx16 acc[NDV];
    float m_ref = NEG_BIG, l_run = 0.f, m_seen = NEG_BIG;
    const float c = kp.scale_log2;
    typedef __attribute__((address_space(3))) bf16x4 *lds_b64_ptr;

    typedef const __attribute__((address_space(3))) bf16x8 *lds_b128_ptr;
    // LDS fragment reads; `half` = 0, 1: the half of 32 entries of the tile the addresses point to.
    // K: chunk ks of this lane's row.  V^T: fragment i = (k-step kk = i / 4, value tile dvt = i % 4), two
    // transpose reads of four keys each.
    auto load_k = [&](int half, int ks) { return *(lds_b128_ptr)(uintptr_t)(k_addr[ks] + half * 32 * RB); };
    auto load_v = [&](int half, int i) {
        const unsigned o = (half * 32 + (i / NDV) * 16) * RB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(uintptr_t)(v_addr[i % NDV] + o));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(uintptr_t)(v_addr[i % NDV] + o + 2 * RB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // the addresses move on to the next stage (K: tile T -> T+1 at the end of iteration T; V one tile behind)
    auto advance_k = [&](int t) {
        const int d = (t & (NSTAGE - 1)) == NSTAGE - 1 ? -(NSTAGE - 1) * STAGE_BYTES : STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) k_addr[ks] += d;
    };
    auto advance_v = [&](int t) {
        const int d = (t & (NSTAGE - 1)) == NSTAGE - 1 ? -(NSTAGE - 1) * STAGE_BYTES : STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < NDV; ++i) v_addr[i] += d;
    };

    struct TileInfo { bool is_rep, full; int e_tile; float bias; };
    auto tile_info = [&](int tl) {
        TileInfo ti;
        ti.is_rep = tl < n_rep_tiles;
        ti.e_tile = ti.is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        ti.bias = ti.is_rep ? kp.bias_log2 : 0.f;
        // every row of this wavefront sees all 64 entries: the steady state
        ti.full = ti.is_rep ? (ti.e_tile + BN <= mt_w_lo) : (ti.e_tile + BN - 1 <= t_wfirst && ti.e_tile >= mt_w_hi * g);
        return ti;
    };
    // boundary tiles: hide what a row must not see
    auto mask_half = [&](floatx16 &sv, const TileInfo &ti, int half) {
        const int e0 = ti.e_tile + half * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int e = e0 + acc_entry(r, G);
            const bool vis = ti.is_rep ? (e < mt_row) : (e >= raw_lo_row && e <= t_row);
            sv[r] = vis ? sv[r] : -INFINITY;
        }
    };
    auto row_max = [&](const floatx16 &sv, float bias) {
        float mx = sv[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sv[r]);
        mx = fmaxf(fmaf(mx, c, bias), NEG_BIG);
        return fmaxf(mx, __shfl_xor(mx, 32, 64));
    };

    // Pass 0 is the normal one: every row fixes its reference at the first entries it sees and never looks at
    // maxima again.  Its probabilities may grow up to 2^100 above that; only if a row sum ends beyond that (or
    // not finite) the workgroup runs pass 1, which finds every row's true maximum (S^T chains alone), and pass
    // 2, the normal pass from those maxima.
    //
    // The normal pass is a software pipeline over halves of 32 entries, scheduled by hand.  Slot H holds
    //     O^T update of half H-1   (8 independent MFMAs)    with the first half of the softmax of half H, then
    //     S^T chain of half H+1    (8 dependent MFMAs)      with the second half of that softmax,
    // so that matrix and vector instructions are mixed evenly wherever the wavefronts of a SIMD happen to be.
    // Iteration T = slots 2T-1 and 2T: the chains read tile T, the O^T updates tile T-1.  One workgroup
    // barrier per iteration: tile T was requested two iterations earlier; every wavefront is then done with
    // tile T-2, whose stage takes tile T+2.  The O^T update comes first in a slot so that the K fragments
    // requested right after the barrier have eight MFMAs to arrive.  LDS fragments travel in rings of four,
    // requested four MFMAs before use (left alone, the compiler issues each read right before its MFMA and
    // waits out the LDS latency every time).
    constexpr int RING = 4;
    constexpr int LOADS_PER_TILE = 2 * NQ;
    for (int pass = 0;; ++pass) {
#pragma unroll
        for (int i = 0; i < NDV; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        l_run = 0.f;
        if (pass == 2) m_ref = m_seen;
        bool ref_missing = pass != 2;                           // wave-uniform: some row has no reference yet
        issue_copy(0);
        if (1 < n_tiles) issue_copy(1);

        if (pass == 1) {                                        // exact row maxima
            m_seen = NEG_BIG;
            for (int tl = 0; tl < n_tiles; ++tl) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
                if (tl + 2 < n_tiles) issue_copy(tl + 2);
                const TileInfo ti = tile_info(tl);
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    floatx16 sv;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sv[r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_k(half, ks), qf[ks], sv, 0, 0, 0);
                    if (!ti.full) mask_half(sv, ti, half);
                    m_seen = fmaxf(m_seen, row_max(sv, ti.bias));
                }
                advance_k(tl);
            }
            if (n_tiles & (NSTAGE - 1)) {
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) k_addr[ks] -= (n_tiles & (NSTAGE - 1)) * STAGE_BYTES;
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            continue;
        }

        floatx16 sacc[2];                                       // S^T of half H lives in sacc[H % 2]
        union Pb { bf16x8 v[2]; bf16x2 p[8]; } pb[2];           // P^T of half H in pb[H % 2]
        bf16x8 kf[RING], vf[RING];
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
        float nb = 0.f;
        // P^T = exp2(S^T * c + bias - reference) in bf16 and its row sums, two S^T registers at a time so that the
        // work can sit between MFMAs.  Accumulator registers 0..7 / 8..15 are the B operands of the two k-steps of
        // the second product as they are.  The sums are taken over the rounded values, the ones the second product
        // sees.  A row that has seen nothing yet has reference -1e30 and only -inf logits: exact zeros.
        auto softmax_pair = [&](int par, int i) {
            bf16x2 pr;
            pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[par][2 * i], c, nb));
            pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sacc[par][2 * i + 1], c, nb));
            // (the empty statements pin the work to this place: otherwise the compiler sinks it past the
            // branches of the next slot, out of the shadow of this slot's MFMAs)
            unsigned bits = __builtin_bit_cast(unsigned, pr);
            asm volatile("" : "+v"(bits));
            pr = __builtin_bit_cast(bf16x2, bits);
            pb[par].p[i] = pr;
            l_run = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l_run, false);
            asm volatile("" : "+v"(l_run));
        };
        // Slot H (par = H % 2), 16 MFMAs with one softmax pair after every second one:
        //   PV: O^T update of half H-1 (V^T of half 1-par of the tile v_addr points to, tile t_v);
        //   SM: softmax of half H, which is half `par` of tile `ti`;
        //   CH: S^T chain of half H+1 (half 1-par of the tile k_addr points to).
        // The last four requests of each ring are for the next slot (`more_v`: it has an O^T update).
        auto slot = [&](auto par_c, auto pv_c, auto sm_c, auto ch_c, const TileInfo &ti, int t_v, bool more_v) {
            constexpr int par = decltype(par_c)::value;
            constexpr bool PV = decltype(pv_c)::value, SM = decltype(sm_c)::value, CH = decltype(ch_c)::value;
            if (SM) {
                if (!ti.full) mask_half(sacc[par], ti, par);
                if (ref_missing) {                              // the first visible entries of a row fix its reference
                    const float mx = row_max(sacc[par], ti.bias);
                    m_ref = (m_ref == NEG_BIG) ? mx : m_ref;
                    ref_missing = __builtin_amdgcn_ballot_w64(m_ref == NEG_BIG) != 0;
                }
                nb = ti.bias - m_ref;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 2 * NDV; ++i) {
                if (PV) {
                    acc[i % NDV] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % RING], pb[1 - par].v[i / NDV], acc[i % NDV], 0, 0, 0);
                    if (i < 2 * NDV - RING) vf[i % RING] = load_v(1 - par, i + RING);
                }
                if (i >= 2 * NDV - RING) {
                    // half H, the next slot's: the second half of the same tile (par == 1) or the first of the next one
                    if (PV && par == 0 && i == 2 * NDV - RING) advance_v(t_v);
                    if (more_v) vf[i % RING] = load_v(par, i - (2 * NDV - RING));
                }
                if (SM && i % 2 == 0) softmax_pair(par, i / 2);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                if (CH) {
                    if (ks == 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) sacc[1 - par][r] = 0.f;
                    }
                    sacc[1 - par] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks % RING], qf[ks], sacc[1 - par], 0, 0, 0);
                    if (ks < NKS - RING) kf[ks % RING] = load_k(1 - par, ks + RING);
                    else if (par == 1) kf[ks % RING] = load_k(1, ks - (NKS - RING));   // next slot's chain: second half of this tile
                }
                if (SM && ks % 2 == 0) softmax_pair(par, 4 + ks / 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // Iteration T: barrier for tile T, copy of tile T+2, slots 2T-1 and 2T.
        auto iteration = [&](int T, auto first_c, auto last_c) {
            constexpr bool FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
            typedef std::integral_constant<bool, !FIRST> not_first;
            typedef std::integral_constant<bool, !LAST> not_last;
            if (!LAST) {
                // this wavefront's share of tile T has landed (the copy of tile T+1 may be pending) ...
                if (T + 1 < n_tiles) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS_PER_TILE) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();                               // ... and everyone's; everyone is done with tile T-2
#pragma unroll
                for (int f = 0; f < RING; ++f) kf[f] = load_k(0, f);
                __builtin_amdgcn_sched_barrier(0);
                if (T + 2 < n_tiles) issue_copy(T + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
            const TileInfo ti_prev = tile_info(FIRST ? 0 : T - 1), ti_cur = tile_info(LAST ? T - 1 : T);
            slot(std::integral_constant<int, 1>(), not_first(), not_first(), not_last(), ti_prev, T - 1, true);
            slot(std::integral_constant<int, 0>(), not_first(), not_last(), not_last(), ti_cur, T - 1, !LAST);
            if (!LAST) advance_k(T);
        };
        iteration(0, std::true_type(), std::false_type());
        for (int T = 1; T < n_tiles; ++T) iteration(T, std::false_type(), std::false_type());
        iteration(n_tiles, std::false_type(), std::true_type());
        if (n_tiles & (NSTAGE - 1)) {                           // back to stage 0 for another pass
            const int back = (n_tiles & (NSTAGE - 1)) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) k_addr[ks] -= back;
#pragma unroll
            for (int i = 0; i < NDV; ++i) v_addr[i] -= back;
        }

        // every wavefront is done with the stages
        if (pass == 0) {
            const float l_chk = l_run + __shfl_xor(l_run, 32, 64);
            if (!__syncthreads_or(!(l_chk <= 0x1p100f))) break;
        } else {
            __syncthreads();
            break;
        }
    }

    // epilogue: normalise, transpose through LDS, store rows of 256 B coalesced
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.f / l_tot;
    constexpr int ORS = RB + 16;
    static_assert(NW * 32 * ORS <= NSTAGE * STAGE_BYTES, "output staging must fit in the stages");
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
    kp.rbs = NW / kp.hw;
    kp.n_qb = (d.L + 32 * kp.rbs - 1) / (32 * kp.rbs);
    kp.n_units = d.B * d.S * (hps / kp.hw);
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    const long grid = (long)kp.n_units * kp.n_qb;
    attn_gqa_kernel<<<(unsigned)grid, 64 * NW, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
