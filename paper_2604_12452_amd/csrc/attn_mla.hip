// bf16 MFMA attention kernel for the MLA widths (d_c = 512, d_R = 64) on gfx950: prefill over the
// condensed context (section 4.3, Eq. 10; per-query partition of appendix A.2) and, with dense = 1,
// plain causal attention in absorbed form (section 3, Eq. 5).
//
// One workgroup = 4 wavefronts = 128 query rows of one (sequence, head); each wavefront owns 32 rows
// and the whole 512-wide output, one wavefront per SIMD with the full 512-register budget:
//   Q^T fragments   144 VGPRs (held for the whole kernel)
//   O^T accumulator 256 AGPRs (16 tiles of 32 value columns x 32 queries)
// Key tiles of 64 entries x 576 columns are copied global -> LDS by direct-to-LDS loads into two
// 73 KB stages (row stride 73 x 16 B: odd in 16-byte units, so row-strided 16-byte reads spread over
// all banks); the copy of tile i+1 runs while tile i is consumed.  A tile is used twice from LDS: all
// 576 columns as keys, the first 512 as values — the absorbed MLA form needs no separate value tile.
//
// Products are computed transposed so that nothing changes lanes between the two MFMA stages:
//   S^T[key, query]  = K Q^T       A = key rows from LDS (16-byte reads), B = Q^T in registers
//   O^T[dv, query]  += V^T P^T     A = V^T through LDS transpose reads,   B = P^T = exp2(S^T - max)
// In the 32x32 accumulator layout lane l holds query l%32, so softmax statistics are per-lane scalars
// and the S^T registers already are the B fragments of the second product when the V^T operand
// enumerates keys in accumulator order.
//
// Softmax reference: each query row fixes its reference maximum at the first key tile it sees and keeps
// it; numerator and denominator use the same reference, so the result does not depend on it, and O^T is
// never rescaled (no vector arithmetic ever touches the 256 accumulation registers inside the loop).
// Exponents are safe while later logits stay within 2^60 of that reference; if one does not, the
// workgroup repeats its pass once with the row maxima it has by then seen as references.
#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define LCA_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define LCA_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int DP = 512, DS = 64, DQK = 576, DV = 512;
constexpr int BM = 128;                 // query rows per workgroup
constexpr int BN = 64;                  // entries per key tile (two 32-entry halves)
constexpr int CPR = 73;                 // 16-byte chunks per LDS row: 64 pool + 8 sel + 1 pad
constexpr int RSB = CPR * 16;           // LDS row stride in bytes
constexpr int STAGE_CHUNKS = BN * CPR;  // 4672 = 73 wave-wide copies of 64 chunks
constexpr int NKS = DQK / 16;           // 36 k-steps of S^T
constexpr int NDV = DV / 32;            // 16 value tiles
constexpr float NEG_BIG = -1.0e30f;     // stands for -inf in the running maximum (keeps exp2 arguments finite)
constexpr float HEADROOM = 60.0f;        // base-2 exponent headroom above the reference before a pass is repeated

struct MlaParams {
    const uint16_t *Q, *POOL, *SEL, *pool_rep, *sel_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, g, w, m, dense, n_qb;
    float scale_log2, bias_log2;
};

// key row held in accumulator register r of lane group G (lanes 32G..32G+31) of a 32x32 tile
__device__ __forceinline__ int acc_row(int r, int G) { return 8 * (r >> 2) + 4 * G + (r & 3); }

// Copy one 64-entry tile into an LDS stage. Entry rows past the segment end are clamped (masked later).
__device__ __forceinline__ void issue_tile_copy(uint4 *stage, const uint16_t *pbase, const uint16_t *sbase, int e0, int seg_end,
                                                int wave, int lane)
{
    for (int i = wave; i < CPR; i += 4) {            // 73 wave-wide copies, 1 KB of LDS each
        const int pos = i * 64 + lane;
        const int r = pos / CPR, c = pos - r * CPR;
        const int e = min(e0 + r, seg_end - 1);
        const uint16_t *src = c < 64 ? pbase + (size_t)e * DP + c * 8 : sbase + (size_t)e * DS + ((c - 64) & 7) * 8;
        __builtin_amdgcn_global_load_lds(LCA_GLB_PTR(src), LCA_LDS_PTR(stage + i * 64), 16, 0, 0);
    }
}

__global__ __launch_bounds__(256) void attn_mla_kernel(const MlaParams kp)
{
    __shared__ __attribute__((aligned(16))) uint4 stage0[STAGE_CHUNKS];
    __shared__ __attribute__((aligned(16))) uint4 stage1[STAGE_CHUNKS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, G = lane >> 5;

    // Workgroup -> (sequence, head, query block): ids with equal id%8 (same XCD under round-robin
    // dispatch) walk the heads of one query block back to back, heaviest blocks first.
    const int xcd = blockIdx.x & 7, kidx = blockIdx.x >> 3;
    const int h = kidx % kp.H;
    const int ord = (kidx / kp.H) * 8 + xcd;
    if (ord >= kp.n_qb * kp.B) return;
    const int b = ord % kp.B;
    const int qb = kp.n_qb - 1 - ord / kp.B;
    const int L = kp.L, H = kp.H, g = kp.g, w = kp.w;
    const int s = h / (H / kp.S);

    const int t0 = qb * BM;
    const int t_last = min(t0 + BM, L) - 1;
    const int t_row = t0 + wave * 32 + n;
    const int t_wfirst = t0 + wave * 32, t_wlast = t_wfirst + 31;

    auto groups_visible = [&](int t) { return (kp.dense || t + 1 <= w) ? 0 : (t + 1 - w) / g; };
    const int mt_row = groups_visible(t_row), raw_lo_row = mt_row * g;
    const int mt_blk_lo = groups_visible(t0), mt_blk_hi = groups_visible(t_last);
    const int mt_w_lo = groups_visible(t_wfirst), mt_w_hi = groups_visible(t_wlast);
    const int raw_lo_blk = mt_blk_lo * g;
    const int n_rep_tiles = (mt_blk_hi + BN - 1) / BN;
    const int n_raw_tiles = (t_last + 1 - raw_lo_blk + BN - 1) / BN;
    const int n_tiles = n_rep_tiles + n_raw_tiles;

    const uint16_t *rep_pool = kp.pool_rep + ((size_t)b * kp.S + s) * kp.m * DP;
    const uint16_t *rep_sel = kp.sel_rep + ((size_t)b * kp.S + s) * kp.m * DS;
    const uint16_t *raw_pool = kp.POOL + (size_t)b * L * DP;
    const uint16_t *raw_sel = kp.SEL + (size_t)b * L * DS;

    auto copy_tile = [&](int tl, uint4 *stage) {
        const bool is_rep = tl < n_rep_tiles;
        const int e0 = is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        issue_tile_copy(stage, is_rep ? rep_pool : raw_pool, is_rep ? rep_sel : raw_sel, e0, is_rep ? mt_blk_hi : t_last + 1, wave, lane);
    };

    // Q^T fragments: lane (n, G) holds Q[t_row, ks*16 + 8G .. +7]
    bf16x8 qf[NKS];
    {
        const uint16_t *qp = kp.Q + (((size_t)b * L + min(t_row, L - 1)) * H + h) * DQK + G * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
    }

    // per-lane LDS byte offsets
    const int k_off = n * RSB + G * 16;                                              // S^T: key row n, 16-byte chunk G
    const int v_off = (4 * G + ((lane & 15) >> 2)) * RSB + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;   // V^T transpose read

    floatx16 acc[NDV];
    float m_ref, l_run, m_seen;              // reference / running sum of this lane's keys / largest logit seen (base 2)
    float m_init = NEG_BIG;
    bool exceeded;
restart:
#pragma unroll
    for (int i = 0; i < NDV; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    m_ref = m_init; l_run = 0.f; m_seen = NEG_BIG; exceeded = false;
    copy_tile(0, stage0);

    for (int tl = 0; tl < n_tiles; ++tl) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's share of tile tl has landed
        __syncthreads();                                   // ... and everyone else's; tile tl-1 is fully consumed
        const char *cur = reinterpret_cast<const char *>((tl & 1) ? stage1 : stage0);
        if (tl + 1 < n_tiles) copy_tile(tl + 1, (tl & 1) ? stage0 : stage1);

        const bool is_rep = tl < n_rep_tiles;
        const int e_tile = is_rep ? tl * BN : raw_lo_blk + (tl - n_rep_tiles) * BN;
        const float bias = is_rep ? kp.bias_log2 : 0.f;

#pragma unroll 1
        for (int half = 0; half < 2; ++half) {
            const int e0 = e_tile + half * 32;
            // skip halves no row of this wavefront can see (wave-uniform)
            const bool none = is_rep ? (e0 >= mt_w_hi) : (e0 > t_wlast || e0 + 32 <= mt_w_lo * g);
            if (none) continue;
            const bool full = is_rep ? (e0 + 32 <= mt_w_lo) : (e0 + 31 <= t_wfirst && e0 >= mt_w_hi * g);
            const char *kbase = cur + half * 32 * RSB;

            // ---- S^T = K Q^T ----
            // Written as inline assembly so that this accumulator is an ordinary vector register tuple: all
            // 256 accumulation registers belong to O^T.  The chain reuses one destination back to back; the
            // wait states an MFMA result needs before ordinary vector instructions read it are spent explicitly.
            floatx16 sacc;
            {
                const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(kbase + k_off);
                asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sacc) : "v"(a0), "v"(qf[0]));
            }
#pragma unroll
            for (int ks = 1; ks < NKS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kbase + k_off + ks * 32);
                asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sacc) : "v"(a), "v"(qf[ks]));
            }
            asm("s_nop 15\n\ts_nop 7" : "+v"(sacc));

            // ---- scaled base-2 logits, mask, maximum ----
            float tmax = NEG_BIG;
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
            m_ref = (m_ref == NEG_BIG) ? tmax : m_ref;       // first visible keys of this row fix its reference
            m_seen = fmaxf(m_seen, tmax);
            exceeded |= tmax > m_ref + HEADROOM;
            // ---- P^T = exp2(S^T - m_ref) as bf16 B fragments (registers 0..7 / 8..15 = two k-steps) ----
            bf16x8 pb[2];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float pv = __builtin_amdgcn_exp2f(sacc[kk * 8 + i] - m_ref);
                    l_run += pv;
                    pb[kk][i] = (__bf16)pv;
                }

            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int dvt = 0; dvt < NDV; ++dvt) {
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const char *vp = kbase + v_off + kk * 16 * RSB + dvt * 64;
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(vp));
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(vp + 8 * RSB));
                    const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    acc[dvt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kk], acc[dvt], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: normalise, transpose through LDS (two passes of 256 value columns), store coalesced ----
    // every wavefront is done with the tile stages; repeat the pass if any row ran out of exponent headroom
    if (__syncthreads_or(exceeded)) {
        m_init = m_seen;
        goto restart;
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.f / l_tot;
    constexpr int ORS = 256 * 2 + 16;                    // staging row stride (bytes)
    static_assert(4 * 32 * ORS <= STAGE_CHUNKS * 16, "output staging must fit in one tile stage");
    char *obuf = reinterpret_cast<char *>(stage0) + wave * 32 * ORS;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int d8 = 0; d8 < 8; ++d8)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                union { bf16x4 h; uint2 u; } o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)(acc[pass * 8 + d8][r4 * 4 + i] * inv);
                *reinterpret_cast<uint2 *>(obuf + n * ORS + (d8 * 32 + 8 * r4 + 4 * G) * 2) = o.u;
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll 4
        for (int r2 = 0; r2 < 16; ++r2) {                // one wave-wide store covers two rows of 512 B
            const int r = r2 * 2 + G, t = t_wfirst + r;
            const uint4 v = *reinterpret_cast<const uint4 *>(obuf + r * ORS + n * 16);
            if (t < L) *reinterpret_cast<uint4 *>(kp.O + (((size_t)b * L + t) * H + h) * DV + pass * 256 + n * 8) = v;
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (kp.lse != nullptr && G == 0 && t_row < L)
        kp.lse[((size_t)b * L + t_row) * H + h] = (m_ref + log2f(l_tot)) * 0.6931471805599453f;
}

}  // namespace

bool attn_mla_supported(const Dims &d) { return d.dtype == LCA_BF16 && d.mode == LCA_MODE_MLA && d.d_pool == DP && d.d_sel == DS; }

hipError_t launch_attn_mla(const AttnArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    MlaParams kp;
    kp.Q = (const uint16_t *)a.Q; kp.POOL = (const uint16_t *)a.POOL; kp.SEL = (const uint16_t *)a.SEL;
    kp.pool_rep = (const uint16_t *)a.pool_rep; kp.sel_rep = (const uint16_t *)a.sel_rep;
    kp.O = (uint16_t *)a.O; kp.lse = a.lse;
    kp.B = d.B; kp.L = d.L; kp.H = d.H; kp.S = d.S; kp.g = d.g; kp.w = d.w; kp.m = d.m; kp.dense = a.dense;
    kp.n_qb = (d.L + BM - 1) / BM;
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    const long units = (long)kp.n_qb * d.B;
    const long grid = ((units + 7) / 8) * 8 * d.H;
    attn_mla_kernel<<<(unsigned)grid, 256, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
