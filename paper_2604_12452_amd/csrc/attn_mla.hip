// bf16 MFMA attention kernel for the MLA widths (d_c = 512, d_R = 64) on gfx950: prefill over the
// condensed context (section 4.3, Eq. 10; per-query partition of appendix A.2) and, with dense = 1,
// plain causal attention in absorbed form (section 3, Eq. 5).
//
// One workgroup = 4 wavefronts = 128 query rows of one (sequence, head); each wavefront owns 32 rows
// and the whole 512-wide output, one wavefront per SIMD with the full 512-register budget:
//   Q^T fragments   144 VGPRs (held for the whole kernel)
//   O^T accumulator 256 AGPRs (16 tiles of 32 value columns x 32 queries)
// Key tiles of 32 entries x 576 columns are copied global -> LDS by direct-to-LDS loads into four
// 36.5 KB stages; copies run three tiles ahead of their use.  A stage holds the latent part as 32 rows
// of 1024 B at a stride of 1040 B and the RoPE part as 32 x 128 B, 16-byte chunks XOR-swizzled by row
// so that one wave-wide load moves eight rows.  S^T row m is computed from LDS row pi(m), a fixed
// permutation inside each half of 16 rows (pi(8h + 4G + j) = 4j + 2h + G): with it both the
// row-strided 16-byte key reads (16 lanes = 16 rows that differ mod 16) and the transpose reads of the
// value operand (each 16-lane block touches 4 rows that are 4 apart) spread over all 64 banks.  A tile is used
// twice from LDS: all 576 columns as keys, the first 512 as values — the absorbed MLA form needs no
// separate value tile.
//
// Products are computed transposed so that nothing changes lanes between the two MFMA stages:
//   S^T[key, query]  = K Q^T       A = key rows from LDS (16-byte reads), B = Q^T in registers
//   O^T[dv, query]  += V^T P^T     A = V^T through LDS transpose reads,   B = P^T = exp2(S^T - ref)
// In the 32x32 accumulator layout lane l holds query l%32, so softmax statistics are per-lane scalars
// and the S^T registers already are the B fragments of the second product when the V^T operand
// enumerates keys in accumulator order.
//
// Software pipeline: while the matrix core runs the S^T chain of tile t+1, the vector ALU turns the
// S^T of tile t into P^T (its instructions are placed between the MFMAs of the chain); then the O^T
// update of tile t runs.  One workgroup barrier per tile.
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

#define LCA_FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int DP = 512, DS = 64, DQK = 576, DV = 512;
constexpr int BM = 128;                 // query rows per workgroup
constexpr int BN = 32;                  // entries per key tile
constexpr int NSTAGE = 4;
constexpr int RSB = 1040;               // LDS row stride of the latent part in bytes: 1024 + 16
constexpr int SEL_OFF = BN * RSB;       // the RoPE part of a stage starts here: 32 rows x 128 B, swizzled
constexpr int STAGE_BYTES = SEL_OFF + BN * DS * 2;   // 37 376
constexpr int COPIES_PER_TILE = 9;      // direct-to-LDS loads one wavefront issues per tile (8 latent rows + 1 RoPE block)
constexpr int NKS = DQK / 16;           // 36 k-steps of S^T
constexpr int NDV = DV / 32;            // 16 value tiles
#ifndef LCA_CHAIN_DEPTH
#define LCA_CHAIN_DEPTH 6
#endif
constexpr int CHAIN_DEPTH = LCA_CHAIN_DEPTH;   // key fragments in flight ahead of the S^T chain
constexpr int MLA_GRID = 256;            // workgroups of the persistent kernel = CUs of the chip
constexpr float NEG_BIG = -1.0e30f;     // stands for -inf in running maxima (keeps exp2 arguments finite)
constexpr float HEADROOM = 60.0f;       // base-2 exponent headroom above the reference before a pass is repeated

struct MlaParams {
    const uint16_t *Q, *POOL, *SEL, *pool_rep, *sel_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, g, w, m, dense, n_qb;
    float scale_log2, bias_log2;
};

// Accumulator register r of lane group G (lanes 32G..32G+31) of a 32x32 tile holds S^T row
// m = 8*(r/4) + 4G + r%4.  S^T row m is computed from LDS row (= tile entry) pi(m): inside each half of 16,
// pi(8h + 4G + j) = 4j + 2h + G.
__device__ __forceinline__ int lds_row_of_m(int m) { return (m & 16) + 4 * (m & 3) + 2 * ((m >> 3) & 1) + ((m >> 2) & 1); }
__device__ __forceinline__ int acc_entry(int r, int G) { return lds_row_of_m(8 * (r >> 2) + 4 * G + (r & 3)); }

// per-lane softmax state (base-2 logits): reference, running sum over this lane's keys, largest seen
struct RowState {
    float m_ref, l_run, m_seen;
    bool exceeded;
};

// Fragments of the V^T operand: two groups of PV_GROUP steps (double-buffered bursts of transpose reads).
// Step j of the O^T update = (value tile j/2, k-step j%2).
#ifndef LCA_PV_GROUP
#define LCA_PV_GROUP 4
#endif
constexpr int PV_GROUP = LCA_PV_GROUP;
struct PvFrags {
    bf16x4 lo[2][PV_GROUP], hi[2][PV_GROUP];
};
__device__ __forceinline__ void pv_load_group(PvFrags &f, const char *vp0, int grp, int buf)
{
    typedef __attribute__((address_space(3))) bf16x4 *lds_b64_ptr;
#pragma unroll
    for (int i = 0; i < PV_GROUP; ++i) {
        const int j = grp * PV_GROUP + i;
        if (j < 2 * NDV) {
            // k-slots i = 4h + j of this step hold keys pi(16kk + 8h + 4G + j) = 16kk + 4j + 2h + G: the lanes of a
            // 16-lane block address rows 4j + G (j = lane bits 2..3, part of vp0); h = 0 / 1 adds two rows
            const char *vp = vp0 + (j & 1) * 16 * RSB + (j >> 1) * 64;
            f.lo[buf][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vp));
            f.hi[buf][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vp + 2 * RSB));
        }
    }
}

// What one wavefront needs to copy its share of a key tile.
struct CopyDesc {
    int e0, last;                 // first entry of the tile, last valid entry of the segment
};
// The same for one wavefront, in the form the copies use: its first row and how far its rows may go.
struct WaveCopy {
    const uint16_t *pool0, *sel0;     // the wavefront's first row of the latent / RoPE part: entry min(e0 + 8*wave, last)
    int dmax;                         // rows 0..dmax after that one exist (>= 0); later ones are clamped to row dmax
};

// One direct-to-LDS load of 64 x 16 bytes: lane l fetches global bytes [base + voff, +16) into LDS bytes
// [lds_addr + 16 l, +16).  Written as inline assembly on purpose: the compiler makes every LDS read that
// follows a direct-to-LDS load it knows about wait for that load, and here the copy must stay in flight
// for two more tiles.  Ordering is kept by hand instead: s_waitcnt vmcnt + workgroup barrier in the tile
// loop before a stage is read, 9 loads per tile and wavefront.
__device__ __forceinline__ void dma_1k(unsigned voff, const void *base, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_addr));   // writes M0, which no compiler-generated instruction of this kernel uses
}

__device__ __forceinline__ unsigned lds_address(const char *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

// `pool` / `sel` = first row of the segment (representatives or raw tokens).
// One of the 9 copies a wavefront makes per tile: j < 8 moves latent row 8*wave + j (1 KB), j == 8 moves the
// RoPE parts of rows 8*wave .. 8*wave+7 (1 KB; lane l fills slot l&7 of local row l>>3 with the chunk
// sel_chunk that the swizzle assigns to that slot).  Rows past the end of the segment are clamped here and
// masked later.
__device__ __forceinline__ WaveCopy wave_copy(const uint16_t *pool, const uint16_t *sel, const CopyDesc &cd, int wave)
{
    WaveCopy wc;
    const int first = cd.e0 + 8 * wave, r0 = min(first, cd.last);     // 0 <= r0 <= last: the base row always exists
    wc.pool0 = pool + (long)r0 * DP;
    wc.sel0 = sel + (long)r0 * DS;
    wc.dmax = max(cd.last - first, 0);                                // all eight rows past the segment: every one reads row `last`
    return wc;
}

// The row offset (0 .. 7 KB; the hardware takes the per-lane offset as unsigned, so it must never be negative)
// travels in the per-lane address offset, so that a row costs a scalar min and shift and one vector add
// instead of 64-bit scalar address arithmetic.
__device__ __forceinline__ void issue_copy_part(int j, const char *stage, const WaveCopy &wc, int wave, int lane, int sel_chunk)
{
    if (j < 8) {
        const int d = min(j, wc.dmax);
        dma_1k(lane * 16 + d * (DP * 2), wc.pool0, lds_address(stage) + (8 * wave + j) * RSB);
    } else {
        const int d = min(lane >> 3, wc.dmax);
        dma_1k(d * (DS * 2) + sel_chunk * 16, wc.sel0, lds_address(stage) + SEL_OFF + 8 * wave * (DS * 2));
    }
}

__device__ __forceinline__ void issue_copy(const char *stage, const uint16_t *pool, const uint16_t *sel, const CopyDesc &cd, int wave, int lane,
                                           int sel_chunk)
{
    const WaveCopy wc = wave_copy(pool, sel, cd, wave);
#pragma unroll
    for (int j = 0; j < COPIES_PER_TILE; ++j) issue_copy_part(j, stage, wc, wave, lane, sel_chunk);
}

// S^T chain of one tile (36 MFMAs into `snext`, key fragments prefetched CHAIN_DEPTH deep) and, when SOFTMAX,
// the vector work that turns the previous tile's S^T (`scur`) into P^T fragments, spread over the
// chain's issue slots.  `kb` = LDS address of this lane's first key fragment of the chain's tile.
// The MFMAs are inline assembly so that their accumulator is an ordinary vector register tuple (all 256
// accumulation registers belong to O^T); the wait states an MFMA result needs before vector
// instructions read it are spent explicitly at the end of the chain.
// When PV_PREFETCH, the copy of a later tile and the first burst of V^T reads of the O^T update that follows are
// issued in the last slots of the chain, and the explicit wait states are left out: the caller keeps every reader of the chain's
// result behind the whole O^T update (see tile_step).
template <bool CHAIN, bool SOFTMAX, bool PV_PREFETCH>
__device__ __forceinline__ void chain_and_softmax(const char *kb, const char *kb_sel, int x6, const bf16x8 (&qf)[NKS], floatx16 &snext,
                                                  const floatx16 &scur, bf16x8 (&pb)[2], RowState &st, float c, float bias, PvFrags &pvf,
                                                  const char *vp0, const char *dma_stage, const WaveCopy &wc, int wave, int lane, int sel_chunk)
{
    // key fragment of k-step ks: latent columns from the row-strided part, RoPE columns (ks >= 32) from the swizzled part
    auto frag = [&](int ks) {
        const char *p = ks < DP / 16 ? kb + ks * 32 : kb_sel + ((x6 ^ (2 * (ks - DP / 16))) << 4);
        return *reinterpret_cast<const bf16x8 *>(p);
    };
    bf16x8 fr[CHAIN_DEPTH];
    if (CHAIN) {
#pragma unroll
        for (int i = 0; i < CHAIN_DEPTH; ++i) fr[i] = frag(i);
    }
    float mx[6], nb = 0.f, p[16];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        LCA_FENCE();
        if (CHAIN) {
            if (ks == 0)
                asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(snext) : "v"(fr[0]), "v"(qf[0]));
            else
                asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(snext) : "v"(fr[ks % CHAIN_DEPTH]), "v"(qf[ks]));
            if (ks + CHAIN_DEPTH < NKS) fr[ks % CHAIN_DEPTH] = frag(ks + CHAIN_DEPTH);
        }
        if (SOFTMAX) {
            // slots 0..4: maxima of triples; 5..7: reduce and scale; 8: partner lane; 9: reference; 10..25: exponentials
            if (ks < 5) mx[ks] = fmaxf(fmaxf(scur[3 * ks], scur[3 * ks + 1]), scur[3 * ks + 2]);
            if (ks == 5) mx[5] = fmaxf(fmaxf(mx[0], mx[1]), mx[2]);
            if (ks == 6) mx[0] = fmaxf(fmaxf(mx[3], mx[4]), scur[15]);
            if (ks == 7) mx[0] = fmaxf(fmaf(fmaxf(mx[5], mx[0]), c, bias), NEG_BIG);
            if (ks == 8) mx[0] = fmaxf(mx[0], __shfl_xor(mx[0], 32, 64));
            if (ks == 9) {
                st.m_ref = (st.m_ref == NEG_BIG) ? mx[0] : st.m_ref;     // first visible keys of this row fix its reference
                st.m_seen = fmaxf(st.m_seen, mx[0]);
                st.exceeded |= mx[0] > st.m_ref + HEADROOM;
                nb = bias - st.m_ref;
            }
            if (ks >= 10 && ks < 26) {
                const int r = ks - 10;
                p[r] = __builtin_amdgcn_exp2f(fmaf(scur[r], c, nb));
                st.l_run += p[r];
                if (r & 1) {
                    pb[r >> 3][(r & 7) - 1] = (__bf16)p[r - 1];
                    pb[r >> 3][r & 7] = (__bf16)p[r];
                }
            }
        }
        // the copy of the tile three steps ahead rides in the chain's last slots, after the softmax work
        if (PV_PREFETCH && ks >= 26 && ks - 26 < COPIES_PER_TILE) issue_copy_part(ks - 26, dma_stage, wc, wave, lane, sel_chunk);
        if (PV_PREFETCH && ks == 35) pv_load_group(pvf, vp0, 0, 0);
    }
    LCA_FENCE();
    if (CHAIN && !PV_PREFETCH) asm("s_nop 15\n\ts_nop 7" : "+v"(snext));
}

// O^T += V^T P^T for one tile; vp0 = this lane's transpose-read address in the tile's stage; group 0 of the
// V^T fragments is already on its way.  The compiler only ever waits for ALL outstanding transpose reads, so
// the reads of the next group go out in one burst right after the first MFMA of the current group and have
// the rest of the group's MFMAs to land.
__device__ __forceinline__ void pv_update(PvFrags &f, const char *vp0, const bf16x8 (&pb)[2], floatx16 (&acc)[NDV])
{
    constexpr int NSTEP = 2 * NDV;
#pragma unroll
    for (int j = 0; j < NSTEP; ++j) {
        const int grp = j / PV_GROUP, i = j % PV_GROUP, buf = grp & 1;
        LCA_FENCE();
        const bf16x8 a = __builtin_shufflevector(f.lo[buf][i], f.hi[buf][i], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[j >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[j & 1], acc[j >> 1], 0, 0, 0);
        if (i == 0 && (grp + 1) * PV_GROUP < NSTEP) {
            LCA_FENCE();
            pv_load_group(f, vp0, grp + 1, buf ^ 1);
        }
    }
    LCA_FENCE();
}

// One pipeline step: copy of tile t+3 (into dma_stage), S^T chain of tile t+1 with the softmax of tile t in
// its shadow, O^T update of tile t.
__device__ __forceinline__ void tile_step(const char *dma_stage, const char *chain_stage, const char *pv_stage, const WaveCopy &wc, int wave,
                                          int lane, int sel_chunk, int k_off, int ksel_off,
                                          int x6, int v_off, const bf16x8 (&qf)[NKS], floatx16 &snext, const floatx16 &scur, bf16x8 (&pb)[2],
                                          RowState &st, float c, float bias, floatx16 (&acc)[NDV])
{
    PvFrags pvf;
    chain_and_softmax<true, true, true>(chain_stage + k_off, chain_stage + ksel_off, x6, qf, snext, scur, pb, st, c, bias, pvf, pv_stage + v_off,
                                        dma_stage, wc, wave, lane, sel_chunk);
    pv_update(pvf, pv_stage + v_off, pb, acc);
    // Anchor: nothing may read the chain's result before this point (the compiler takes an inline-assembly
    // result as ready at once; the 32 MFMAs of the O^T update are the wait states it actually needs).
    asm("" : "+v"(snext));
    LCA_FENCE();
}

// Everything one workgroup needs to know about one work item = 128 query rows of one (sequence, head).
struct Blk {
    int b, h, t0, t_last;                    // sequence, head, first / last query row
    int t_row, mt_row, raw_lo_row;           // per lane: query row, representatives it sees, first raw token it sees
    int raw_lo_blk, mt_blk_hi;               // first raw token / representatives any row of the block sees
    int n_rep_tiles, n_tiles;
    int rep_full_end, raw_full_lo, raw_full_hi;   // tiles this wavefront sees completely (no masking)
    const uint16_t *rep_pool, *rep_sel, *raw_pool, *raw_sel;
};

__device__ __forceinline__ Blk make_blk(const MlaParams &kp, int b, int h, int qb, int wave, int n)
{
    Blk k;
    const int L = kp.L, g = kp.g, w = kp.w;
    auto groups_visible = [&](int t) { return (kp.dense || t + 1 <= w) ? 0 : (t + 1 - w) / g; };
    k.b = b; k.h = h;
    k.t0 = qb * BM;
    k.t_last = min(k.t0 + BM, L) - 1;
    const int t_wfirst = k.t0 + wave * 32, t_wlast = t_wfirst + 31;
    k.t_row = t_wfirst + n;
    k.mt_row = groups_visible(k.t_row);
    k.raw_lo_row = k.mt_row * g;
    const int mt_blk_lo = groups_visible(k.t0), mt_w_lo = groups_visible(t_wfirst), mt_w_hi = groups_visible(t_wlast);
    k.mt_blk_hi = groups_visible(k.t_last);
    k.raw_lo_blk = mt_blk_lo * g;
    k.n_rep_tiles = (k.mt_blk_hi + BN - 1) / BN;
    k.n_tiles = k.n_rep_tiles + (k.t_last + 1 - k.raw_lo_blk + BN - 1) / BN;
    k.rep_full_end = mt_w_lo / BN;
    k.raw_full_lo = k.n_rep_tiles + (mt_w_hi * g - k.raw_lo_blk + BN - 1) / BN;
    k.raw_full_hi = k.n_rep_tiles + max(0, (t_wfirst + 1 - k.raw_lo_blk) / BN);
    const int s = h / (kp.H / kp.S);
    k.rep_pool = kp.pool_rep + ((size_t)b * kp.S + s) * kp.m * DP;
    k.rep_sel = kp.sel_rep + ((size_t)b * kp.S + s) * kp.m * DS;
    k.raw_pool = kp.POOL + (size_t)b * L * DP;
    k.raw_sel = kp.SEL + (size_t)b * L * DS;
    return k;
}

__device__ __forceinline__ CopyDesc copy_desc(const Blk &k, int tl)
{
    const bool is_rep = tl < k.n_rep_tiles;
    CopyDesc cd;
    cd.e0 = is_rep ? tl * BN : k.raw_lo_blk + (tl - k.n_rep_tiles) * BN;
    cd.last = (is_rep ? k.mt_blk_hi : k.t_last + 1) - 1;
    return cd;
}

// copies of tiles 0..2 of a work item into stages 0..2 (past the last tile: that tile again, nobody reads it)
__device__ __forceinline__ void issue_first_copies(const Blk &k, char (*stages)[STAGE_BYTES], int wave, int lane, int sel_chunk)
{
    for (int tl = 0; tl < 3; ++tl) {
        const int tc = min(tl, k.n_tiles - 1);
        issue_copy(stages[tl], tc < k.n_rep_tiles ? k.rep_pool : k.raw_pool, tc < k.n_rep_tiles ? k.rep_sel : k.raw_sel, copy_desc(k, tc), wave,
                   lane, sel_chunk);
    }
}

// Q^T fragments of a work item: lane (n, G) holds Q[t_row, ks*16 + 8G .. +7]
__device__ __forceinline__ void load_q(const MlaParams &kp, const Blk &k, int G, bf16x8 (&qf)[NKS])
{
    const uint16_t *qp = kp.Q + (((size_t)k.b * kp.L + min(k.t_row, kp.L - 1)) * kp.H + k.h) * DQK + G * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
}

// Persistent kernel: one workgroup per CU walks a list of work items.  Workgroup w lives on XCD w%8 (round-
// robin placement) and is slot w/8 of that XCD; the XCD's item list is (query-block order x, x+8, ... of
// the heaviest-first order) x (all heads), so that at any time the slots of an XCD work on the heads of
// one or two query blocks and share their K/V tiles in that XCD's L2.  The next item's queries and first
// tiles are requested before the current item's output is written, so the transition costs no round trip.
__global__ __launch_bounds__(256) void attn_mla_kernel(const MlaParams kp)
{
    __shared__ __attribute__((aligned(1024))) char stages[NSTAGE][STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, G = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = kp.L, H = kp.H;

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, n_slots = gridDim.x >> 3;
    const int n_units = kp.n_qb * kp.B;                       // (query block, sequence) pairs, heaviest first
    const int items_per_xcd = ((n_units + 7) / 8) * H;        // some may fall past n_units
    auto item = [&](int kidx, int &b, int &h, int &qb) {      // false when the item does not exist
        h = kidx % H;
        const int ord = (kidx / H) * 8 + xcd;
        b = ord % kp.B;
        qb = kp.n_qb - 1 - ord / kp.B;
        return kidx < items_per_xcd && ord < n_units;
    };

    // per-lane LDS byte offsets
    const int krow = lds_row_of_m(n);                                                // LDS row behind S^T row n
    const int k_off = krow * RSB + G * 16;                                           // S^T, latent part: 16-byte chunk G of that row
    const int xs = (krow >> 1) & 7;                                                  // swizzle of that row in the RoPE part
    const int ksel_off = SEL_OFF + krow * (DS * 2) + ((G ^ (xs & 1)) << 4);          // S^T, RoPE part: chunk (2j+G) sits at slot (2j+G)^xs
    const int x6 = xs & 6;
    const int v_off = (4 * ((lane & 15) >> 2) + G) * RSB + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;   // V^T transpose read
    // copy side of the swizzle: lane l of the RoPE copy fills slot l&7 of local row l>>3 (row 8*wave + (l>>3) of the tile)
    const int sel_chunk = (lane & 7) ^ ((4 * wave + (lane >> 4)) & 7);
    const float c = kp.scale_log2;

    int kidx = slot, ib, ih, iqb;
    while (kidx < items_per_xcd && !item(kidx, ib, ih, iqb)) kidx += n_slots;   // items past n_units only sit at the list's end
    if (kidx >= items_per_xcd) return;
    Blk cur = make_blk(kp, ib, ih, iqb, wave, n);

    bf16x8 qf[NKS];
    floatx16 acc[NDV];
    RowState st;
    issue_first_copies(cur, stages, wave, lane, sel_chunk);
    load_q(kp, cur, G, qf);

    while (true) {
        float m_init = NEG_BIG;
    restart:
#pragma unroll
        for (int i = 0; i < NDV; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        st.m_ref = m_init; st.l_run = 0.f; st.m_seen = NEG_BIG; st.exceeded = false;

        // the first tiles and the queries of this item are on their way; then the S^T chain of tile 0
        floatx16 snext, scur;
        bf16x8 pb[2];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        {
            PvFrags unused;
            chain_and_softmax<true, false, false>(stages[0] + k_off, stages[0] + ksel_off, x6, qf, snext, snext, pb, st, c, 0.f, unused, nullptr,
                                                  nullptr, WaveCopy(), wave, lane, sel_chunk);
        }

        for (int tl = 0; tl < cur.n_tiles; ++tl) {
            // everything that does not need the barrier comes before it, so that the chain starts right after it
            const bool is_rep = tl < cur.n_rep_tiles;
            const float bias = is_rep ? kp.bias_log2 : 0.f;
            scur = snext;
            const bool full = tl < cur.rep_full_end || (tl >= cur.raw_full_lo && tl < cur.raw_full_hi);
            if (!full) {   // boundary tiles: hide the entries this row must not see
                const int e0 = is_rep ? tl * BN : cur.raw_lo_blk + (tl - cur.n_rep_tiles) * BN;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int e = e0 + acc_entry(r, G);
                    const bool vis = is_rep ? (e < cur.mt_row) : (e >= cur.raw_lo_row && e <= cur.t_row);
                    scur[r] = vis ? scur[r] : -INFINITY;
                }
            }
            // The chain and the copy always run: past the last tile they redo that tile (S^T that nobody reads, a
            // copy into a stage that nobody reads again), which keeps the loop body branch-free.
            const char *dma_stage = stages[(tl + 3) & (NSTAGE - 1)];
            const char *chain_stage = stages[min(tl + 1, cur.n_tiles - 1) & (NSTAGE - 1)], *pv_stage = stages[tl & (NSTAGE - 1)];
            const int tc = min(tl + 3, cur.n_tiles - 1);
            const WaveCopy wc = wave_copy(tc < cur.n_rep_tiles ? cur.rep_pool : cur.raw_pool, tc < cur.n_rep_tiles ? cur.rep_sel : cur.raw_sel,
                                          copy_desc(cur, tc), wave);
            // tile tl+1 has landed: its copy was issued two iterations ago, only tile tl+2's 9 loads may be pending ...
            asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
            __syncthreads();      // ... for every wavefront, and every wavefront is done with tile tl-1
            tile_step(dma_stage, chain_stage, pv_stage, wc, wave, lane, sel_chunk, k_off, ksel_off, x6, v_off, qf, snext, scur, pb, st, c, bias,
                      acc);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the trailing copies have landed before the stages are reused
        // every wavefront is done with the tile stages; repeat the pass if any row ran out of exponent headroom
        if (__syncthreads_or(st.exceeded)) {
            m_init = st.m_seen;
            issue_first_copies(cur, stages, wave, lane, sel_chunk);
            goto restart;
        }

        // request the next item's first tiles (stages 0..2) and queries before writing this item's output
        int nb, nh, nqb;
        kidx += n_slots;
        const bool has_next = item(kidx, nb, nh, nqb);
        const int out_b = cur.b, out_h = cur.h, out_t0 = cur.t0, out_t_row = cur.t_row;
        if (has_next) {
            cur = make_blk(kp, nb, nh, nqb, wave, n);
            issue_first_copies(cur, stages, wave, lane, sel_chunk);
            load_q(kp, cur, G, qf);
        }

        // ---- epilogue: normalise, transpose through LDS stage 3 (four passes of 128 value columns), store coalesced ----
        const float l_tot = st.l_run + __shfl_xor(st.l_run, 32, 64);
        const float inv = 1.f / l_tot;
        constexpr int ORS = 128 * 2 + 16;                    // staging row stride (bytes)
        static_assert(4 * 32 * ORS <= STAGE_BYTES, "output staging must fit in one tile stage");
        char *obuf = &stages[3][0] + wave * 32 * ORS;
        const int t_wfirst = out_t0 + wave * 32;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
#pragma unroll
            for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    union { bf16x4 h; uint2 u; } o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o.h[i] = (__bf16)(acc[pass * 4 + d4][r4 * 4 + i] * inv);
                    *reinterpret_cast<uint2 *>(obuf + n * ORS + (d4 * 32 + 8 * r4 + 4 * G) * 2) = o.u;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r4 = 0; r4 < 8; ++r4) {                 // one wave-wide store covers four rows of 256 B
                const int r = r4 * 4 + (lane >> 4), t = t_wfirst + r;
                const uint4 v = *reinterpret_cast<const uint4 *>(obuf + r * ORS + (lane & 15) * 16);
                if (t < L) *reinterpret_cast<uint4 *>(kp.O + (((size_t)out_b * L + t) * H + out_h) * DV + pass * 128 + (lane & 15) * 8) = v;
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (kp.lse != nullptr && G == 0 && out_t_row < L)
            kp.lse[((size_t)out_b * L + out_t_row) * H + out_h] = (st.m_ref + log2f(l_tot)) * 0.6931471805599453f;
        if (!has_next) break;
    }
}

}  // namespace

bool attn_mla_supported(const Dims &d)
{
    return d.dtype == LCA_BF16 && d.mode == LCA_MODE_MLA && d.d_pool == DP && d.d_sel == DS && d.scale > 0.f;
}

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
    // persistent grid: one workgroup per CU (a workgroup takes all of a CU's LDS and registers)
    const long items = (((long)kp.n_qb * d.B + 7) / 8) * 8 * d.H;
    long grid = items < MLA_GRID ? items : MLA_GRID;
    grid = (grid + 7) / 8 * 8;
    attn_mla_kernel<<<(unsigned)grid, 256, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
