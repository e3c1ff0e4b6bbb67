// bf16 / fp16 MFMA attention kernel for the MLA widths (d_c = 512, d_R = 64) on gfx950: prefill over the
// condensed context (section 4.3, Eq. 10; per-query partition of appendix A.2) and, with dense = 1,
// plain causal attention in absorbed form (section 3, Eq. 5).
//
// One workgroup = 4 wavefronts = 128 query rows of one (sequence, head); each wavefront owns 32 rows
// and the whole 512-wide output, one wavefront per SIMD with the full 512-register budget:
//   Q^T fragments   144 VGPRs (held for a whole work item)
//   O^T accumulator 256 AGPRs (16 tiles of 32 value columns x 32 queries)
// Key tiles of 32 entries x 576 columns are copied global -> LDS by direct-to-LDS loads into four
// 36.5 KB stages; copies run three tiles ahead of their use.  A stage holds the latent part as 32 rows
// of 1024 B at a stride of 1040 B and the RoPE part as 32 x 128 B, 16-byte chunks XOR-swizzled by row
// so that one wave-wide load moves eight rows.  S^T row m is computed from LDS row pi(m), a fixed
// permutation inside each half of 16 rows (pi(8h + 4G + j) = 4j + 2h + G): with it both the
// row-strided 16-byte key reads (16 lanes = 16 rows that differ mod 16) and the transpose reads of the
// value operand (each 16-lane block touches 4 rows that are 4 apart) spread over all 64 banks.  A tile is used
// twice from LDS: all 576 columns as keys, the first 512 as values -- the absorbed MLA form needs no
// separate value tile.
//
// Products are computed transposed so that nothing changes lanes between the two MFMA stages:
//   S^T[key, query]  = K Q^T       A = key rows from LDS (16-byte reads), B = Q^T in registers
//   O^T[dv, query]  += V^T P^T     A = V^T through LDS transpose reads,   B = P^T = exp2(S^T - ref)
// In the 32x32 accumulator layout lane l holds query l%32, so softmax statistics are per-lane scalars
// and the S^T registers already are the B fragments of the second product when the V^T operand
// enumerates keys in accumulator order.
//
// With one wavefront per SIMD every instruction the wavefront issues costs about five cycles of its
// time (nine for an exponential), and an MFMA occupies the matrix core for 32: the loop is written so
// that each MFMA is followed by at most five or six other instructions.  Software pipeline, one workgroup
// barrier per tile: after the barrier of iteration t the wavefront requests the first key fragments of
// tile t+1 and meanwhile runs the last four MFMAs of the O^T update of tile t-1 (their V^T fragments are
// already in registers); then the S^T chain of tile t+1 (36 MFMAs) with the softmax of tile t between
// its MFMAs and the copy of tile t+3 in its last slots; then the O^T update of tile t (28 MFMAs), whose
// free issue slots take the loop's scalar bookkeeping for iteration t+1, a few instructions per MFMA.
//
// Softmax reference: each query row fixes its reference at the first entries it sees and never looks at
// maxima again; numerator and denominator use the same reference, so the result does not depend on it,
// and O^T is never rescaled (no vector arithmetic touches the 256 accumulation registers inside the
// loop).  If a row sum ends beyond 2^90 (or not finite) the workgroup finds every row's exact maximum in
// a pass of S^T chains alone and runs the item again from those.
#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// fp16 runs through the same code (template parameter F16): fragments travel in the bf16 vector types as plain 16-bit
// containers, and only the matrix instructions, the two conversions (P^T, output) and the softmax range differ.
union Pb { bf16x8 v[2]; bf16x2 p[8]; };     // P^T of one tile: the B operands of the two k-steps of the second product
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const char *lds_cptr;

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
constexpr int DU = 128;                  // UP variant: width of a head's value after the up-projection
constexpr float NEG_BIG = -1.0e30f;     // stands for -inf in running maxima (keeps exp2 arguments finite)
constexpr float L_LIMIT = 0x1p90f;      // a row sum beyond this (or not finite) makes the workgroup repeat the item from exact maxima
// fp16 ends at 65504: the fp16 kernels keep the largest exponential of each row (one v_max3 per pair) and repeat the item
// from exact maxima if it left the type's range.  The reference sits 4 binades above the first maximum a row sees
// (first entries at 2^-4): later logits may be 2^19 times larger before that happens, at the price of 4 of fp16's 24
// binades at the bottom.
constexpr float P_LIMIT_F16 = 65000.f;
constexpr float REF_SHIFT_F16 = 4.f;

struct MlaParams {
    const uint16_t *Q, *POOL, *SEL, *pool_rep, *sel_rep;
    uint16_t *O;
    float *lse;
    const uint16_t *W_up;   // UP variant: value up-projection W^UV in fragment order (pack_up_kernel), and O is [B, L, H, DU]
    int B, L, H, S, g, w, m, dense, n_qb;
    float scale_log2, bias_log2;
};

// Accumulator register r of lane group G (lanes 32G..32G+31) of a 32x32 tile holds S^T row
// m = 8*(r/4) + 4G + r%4.  S^T row m is computed from LDS row (= tile entry) pi(m): inside each half of 16,
// pi(8h + 4G + j) = 4j + 2h + G.
__device__ __forceinline__ constexpr int lds_row_of_m(int m) { return (m & 16) + 4 * (m & 3) + 2 * ((m >> 3) & 1) + ((m >> 2) & 1); }
__device__ __forceinline__ constexpr int acc_entry(int r, int G) { return lds_row_of_m(8 * (r >> 2) + 4 * G + (r & 3)); }

// per-lane softmax state (base-2 logits): reference and running sum over this lane's keys
struct RowState {
    float m_ref, l_run;
    float p_max;        // fp16 only: the largest exponential of the row so far
};

// Fragments of the V^T operand: a ring of 2*PV_GROUP steps, requested PV_GROUP steps ahead of their use.
// Step j of the O^T update = (value tile j/2, k-step j%2).
#ifndef LCA_PV_GROUP
#define LCA_PV_GROUP 4
#endif
constexpr int PV_GROUP = LCA_PV_GROUP;
struct PvFrags {
    bf16x4 lo[2][PV_GROUP], hi[2][PV_GROUP];
};
// Requests the V^T fragment of step j into its ring slot (steps j and j + 2*PV_GROUP share one).
__device__ __forceinline__ void pv_load_step(PvFrags &f, lds_cptr vp0, int j)
{
    typedef __attribute__((address_space(3))) bf16x4 *lds_b64_ptr;
    const int buf = (j / PV_GROUP) & 1, i = j % PV_GROUP;
    // k-slots i = 4h + j of this step hold keys pi(16kk + 8h + 4G + j) = 16kk + 4j + 2h + G: the lanes of a
    // 16-lane block address rows 4j + G (j = lane bits 2..3, part of vp0); h = 0 / 1 adds two rows
    lds_cptr vp = vp0 + (j & 1) * 16 * RSB + (j >> 1) * 64;
    f.lo[buf][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vp));
    f.hi[buf][i] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(vp + 2 * RSB));
}

// Tile copies go through raw buffer descriptors (base, size in bytes) so that rows past the end of a segment
// need no clamping: the hardware range check turns them into zeros (such entries are masked anyway).
struct Seg {
    unsigned lo, hi, bytes;       // descriptor words 0..2: address bits 0..31, bits 32..47 (stride 0), size
};
__device__ __forceinline__ Seg make_seg(const void *p, long bytes)
{
    const unsigned long long a = (unsigned long long)p;
    return Seg{(unsigned)a, (unsigned)(a >> 32) & 0xFFFFu, (unsigned)bytes};
}
constexpr int RSRC_WORD3 = 0x00020000;   // raw buffer of dwords, gfx9 layout

// What one wavefront needs to copy its 8 rows of one key tile into one stage (all wavefront-uniform).
struct CopyCtl {
    int4v pool_rs, sel_rs;               // descriptors of the latent / RoPE part of the tile's segment
    unsigned soff_lo, soff_hi, soff_sel; // byte offsets of the wavefront's rows 0 and 4 (latent) and row 0 (RoPE) in the segment
    unsigned m0_pool, m0_sel;            // LDS addresses of the wavefront's first row in the stage
};

// One direct-to-LDS load of 64 x 16 bytes: lane l fetches segment bytes [soff + IMM + voff, +16) into LDS bytes
// [m0 + IMM + 16 l, +16) (the instruction offset moves both sides).  Inline assembly on purpose: the compiler
// makes every LDS read that follows a direct-to-LDS load it knows about wait for that load, and here the
// copy must stay in flight for two more tiles.  Ordering is kept by hand instead: s_waitcnt vmcnt + workgroup
// barrier in the tile loop before a stage is read, 9 loads per tile and wavefront.
template <int M0_ADD, int IMM>
__device__ __forceinline__ void dma_1k(unsigned voff, const int4v &rs, unsigned soff, unsigned m0_base)
{
    asm volatile("s_add_u32 m0, %2, %4\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %3 offen offset:%5 lds"
                 : : "v"(voff), "s"(rs), "s"(m0_base), "s"(soff), "n"(M0_ADD), "n"(IMM) : "scc", "memory");   // writes M0, which no compiler-generated instruction of this kernel uses
}

__device__ __forceinline__ unsigned lds_address(const void *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

// One of the 9 copies a wavefront makes per tile: J < 8 moves latent row 8*wave + J (1 KB; LDS rows are RSB
// apart, the instruction offset (J%4) KB already moves the LDS side by as much), J == 8 moves the RoPE parts
// of rows 8*wave .. 8*wave+7 (1 KB; lane l fills slot l&7 of local row l>>3 with the chunk the swizzle assigns
// to that slot: voff_sel = (l>>3)*128 + chunk*16).
template <int J>
__device__ __forceinline__ void issue_copy_part(const CopyCtl &c, unsigned voff_pool, unsigned voff_sel)
{
    if constexpr (J < 4) dma_1k<J * RSB - J * 1024, J * 1024>(voff_pool, c.pool_rs, c.soff_lo, c.m0_pool);
    else if constexpr (J < 8) dma_1k<J * RSB - (J - 4) * 1024, (J - 4) * 1024>(voff_pool, c.pool_rs, c.soff_hi, c.m0_pool);
    else dma_1k<0, 0>(voff_sel, c.sel_rs, c.soff_sel, c.m0_sel);
}
template <int J>
__device__ __forceinline__ void issue_copy_from(const CopyCtl &c, unsigned voff_pool, unsigned voff_sel)
{
    if constexpr (J < COPIES_PER_TILE) {
        issue_copy_part<J>(c, voff_pool, voff_sel);
        issue_copy_from<J + 1>(c, voff_pool, voff_sel);
    }
}

__device__ __forceinline__ void issue_copy_part_dyn(int j, const CopyCtl &c, unsigned voff_pool, unsigned voff_sel)
{
    switch (j) {      // j is a constant after unrolling
    case 0: issue_copy_part<0>(c, voff_pool, voff_sel); break;
    case 1: issue_copy_part<1>(c, voff_pool, voff_sel); break;
    case 2: issue_copy_part<2>(c, voff_pool, voff_sel); break;
    case 3: issue_copy_part<3>(c, voff_pool, voff_sel); break;
    case 4: issue_copy_part<4>(c, voff_pool, voff_sel); break;
    case 5: issue_copy_part<5>(c, voff_pool, voff_sel); break;
    case 6: issue_copy_part<6>(c, voff_pool, voff_sel); break;
    case 7: issue_copy_part<7>(c, voff_pool, voff_sel); break;
    default: issue_copy_part<8>(c, voff_pool, voff_sel); break;
    }
}

// S^T chain of one tile (36 MFMAs into `snext`, key fragments prefetched CHAIN_DEPTH deep) and, when SOFTMAX,
// the vector work that turns the previous tile's S^T (`scur`) into P^T fragments, spread over the
// chain's issue slots.  `kb` / `ksel` = LDS addresses of this lane's key fragments in the chain's tile (latent part: first one; RoPE part: all four).
// The MFMAs are inline assembly so that their accumulator is an ordinary vector register tuple (all 256
// accumulation registers belong to O^T); the wait states an MFMA result needs before vector
// instructions read it are spent explicitly at the end of the chain.
// When PIPELINED, the first key fragments were requested by the caller (chain_prefetch), the copy of a later tile
// and the first burst of V^T reads of the O^T update that follows are issued in the last slots of the chain, and
// the explicit wait states are left out: the caller keeps every reader of the chain's result behind MFMAs of
// the O^T update.
struct ChainFrags { bf16x8 fr[CHAIN_DEPTH]; };
// LDS addresses of this lane's four key fragments of the RoPE part (k-steps 32..35) of a stage: chunk 2j + G of the
// lane's row sits at slot (2j + G) ^ xs.  `first` = address of the slot of j = 0 (x6 = xs & 6 already applied);
// slot bits 1..2 are address bits 5..6, which are zero in the row's base address, so j enters as an exclusive or.
struct KSel { unsigned a[4]; };
__device__ __forceinline__ KSel make_ksel(unsigned first)
{
    return KSel{{first, first ^ (1u << 5), first ^ (2u << 5), first ^ (3u << 5)}};
}
__device__ __forceinline__ bf16x8 chain_frag(lds_cptr kb, const KSel &ksel, int ks)
{
    // key fragment of k-step ks: latent columns from the row-strided part, RoPE columns (ks >= 32) from the swizzled part
    lds_cptr p = ks < DP / 16 ? kb + ks * 32 : (lds_cptr)(uintptr_t)ksel.a[ks - DP / 16];
    return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8 *>(p);
}
__device__ __forceinline__ void chain_prefetch(ChainFrags &cf, lds_cptr kb, const KSel &ksel)
{
#pragma unroll
    for (int i = 0; i < CHAIN_DEPTH; ++i) cf.fr[i] = chain_frag(kb, ksel, i);
}
template <bool SOFTMAX, bool PIPELINED, bool F16>
__device__ __forceinline__ void chain_and_softmax(ChainFrags &cf, lds_cptr kb, const KSel &ksel, const bf16x8 (&qf)[NKS], floatx16 &snext,
                                                  const floatx16 &scur, Pb &pb, RowState &st, float c, float bias, PvFrags &pvf,
                                                  lds_cptr vp0, const CopyCtl &cc, unsigned voff_pool, unsigned voff_sel)
{
    float nb = 0.f, pf[2];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        LCA_FENCE();
        if (ks == 0) {
            if (F16) asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(snext) : "v"(cf.fr[0]), "v"(qf[0]));
            else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(snext) : "v"(cf.fr[0]), "v"(qf[0]));
        } else {
            if (F16) asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(snext) : "v"(cf.fr[ks % CHAIN_DEPTH]), "v"(qf[ks]));
            else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(snext) : "v"(cf.fr[ks % CHAIN_DEPTH]), "v"(qf[ks]));
        }
        LCA_FENCE();        // the MFMA first, then this slot's other work (left alone, the scheduler sometimes puts the MFMA last)
        if (ks + CHAIN_DEPTH < NKS) cf.fr[ks % CHAIN_DEPTH] = chain_frag(kb, ksel, ks + CHAIN_DEPTH);
        if (SOFTMAX) {
            // P^T = exp2(S^T * c + bias - reference), two S^T registers per three slots: an exponential in each of two
            // slots, then the pair is added to the row sum and rounded to bf16.  No maxima here: the reference was
            // fixed when the row saw its first entries.  A row that has seen nothing yet has reference -1e30 and
            // only -inf logits: exact zeros.
            if (ks == 0) nb = bias - st.m_ref;
            if (ks < 24) {
                const int k = ks / 3, sub = ks % 3;
                if (sub < 2) pf[sub] = __builtin_amdgcn_exp2f(fmaf(scur[2 * k + sub], c, nb));
                else {
                    unsigned bits;
                    if (F16) bits = __builtin_bit_cast(unsigned, f16x2{(_Float16)pf[0], (_Float16)pf[1]});
                    else bits = __builtin_bit_cast(unsigned, bf16x2{(__bf16)pf[0], (__bf16)pf[1]});
                    asm volatile("" : "+v"(bits));      // (pins the conversion to this slot: the compiler would gather four of them where the fragment is complete)
                    pb.p[k] = __builtin_bit_cast(bf16x2, bits);
                    if (F16) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(st.p_max) : "v"(pf[0]), "v"(pf[1]));
                    st.l_run += pf[0];       // (two plain additions: v_dot2c_f32_bf16 stalls next to MFMAs, about 25 cycles each)
                    st.l_run += pf[1];
                }
            }
        }
        // the copy of the tile three steps ahead rides in the chain's last slots, after the softmax work
        if (PIPELINED && ks >= 24 && ks - 24 < COPIES_PER_TILE) issue_copy_part_dyn(ks - 24, cc, voff_pool, voff_sel);
        // the V^T fragments of the first steps of the O^T update that follows
        if (PIPELINED && ks >= NKS - PV_GROUP) pv_load_step(pvf, vp0, ks - (NKS - PV_GROUP));
    }
    LCA_FENCE();
    if (!PIPELINED) asm("s_nop 15\n\ts_nop 7" : "+v"(snext));
}

constexpr int PV_STEPS = 2 * NDV;                 // 32 MFMAs of the O^T update of one tile
constexpr int PV_TAIL = PV_GROUP;                 // the last group is held back: it runs after the next barrier
constexpr int PV_NGROUPS = PV_STEPS / PV_GROUP;
static_assert((PV_NGROUPS & 1) == 0, "the held-back group must sit in buffer 1");

// O^T += V^T P^T for one tile, all but the last group of steps; vp0 = this lane's transpose-read address in the
// tile's stage; the V^T fragments of the first PV_GROUP steps are already on their way, every step requests the
// fragment of the step PV_GROUP later.  `shadow(j)` is work for the issue slots that the MFMAs leave free.  The
// last group's fragments are left in buffer 1 for pv_tail.
template <bool F16>
__device__ __forceinline__ floatx16 pv_mfma(const bf16x8 &a, const bf16x8 &b, const floatx16 &c)
{
    if (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
template <bool F16, class Shadow>
__device__ __forceinline__ void pv_update(PvFrags &f, lds_cptr vp0, const Pb &pb, floatx16 (&acc)[NDV], Shadow shadow)
{
#pragma unroll
    for (int j = 0; j < PV_STEPS - PV_TAIL; ++j) {
        const int grp = j / PV_GROUP, i = j % PV_GROUP, buf = grp & 1;
        LCA_FENCE();
        const bf16x8 a = __builtin_shufflevector(f.lo[buf][i], f.hi[buf][i], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[j >> 1] = pv_mfma<F16>(a, pb.v[j & 1], acc[j >> 1]);
        LCA_FENCE();
        pv_load_step(f, vp0, j + PV_GROUP);
        LCA_FENCE();
        shadow(j);
    }
    LCA_FENCE();
}
// The held-back steps of the previous tile's O^T update: their fragments are in registers, so they run while
// the first key fragments of the next S^T chain travel from LDS.
template <bool F16>
__device__ __forceinline__ void pv_tail(const PvFrags &f, const Pb &pb, floatx16 (&acc)[NDV])
{
#pragma unroll
    for (int j = PV_STEPS - PV_TAIL; j < PV_STEPS; ++j) {
        const int i = j % PV_GROUP;
        LCA_FENCE();
        const bf16x8 a = __builtin_shufflevector(f.lo[1][i], f.hi[1][i], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[j >> 1] = pv_mfma<F16>(a, pb.v[j & 1], acc[j >> 1]);
    }
    LCA_FENCE();
}

// Everything one workgroup needs to know about one work item = 128 query rows of one (sequence, head).
struct Blk {
    int b, h, t0, t_last;                    // sequence, head, first / last query row
    int t_row, mt_row, raw_lo_row;           // per lane: query row, representatives it sees, first raw token it sees
    int raw_lo_blk, mt_blk_hi;               // first raw token / representatives any row of the block sees
    int n_rep_tiles, n_tiles;
    int rep_full_end, raw_full_lo, raw_full_hi;   // tiles this wavefront sees completely (no masking)
    Seg rep_pool, rep_sel, raw_pool, raw_sel;     // the two segments: visible representatives, raw tokens 0 .. t_last of the sequence
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
    k.rep_pool = make_seg(kp.pool_rep + ((size_t)b * kp.S + s) * kp.m * DP, (long)k.mt_blk_hi * (DP * 2));
    k.rep_sel = make_seg(kp.sel_rep + ((size_t)b * kp.S + s) * kp.m * DS, (long)k.mt_blk_hi * (DS * 2));
    k.raw_pool = make_seg(kp.POOL + (size_t)b * L * DP, (long)(k.t_last + 1) * (DP * 2));
    k.raw_sel = make_seg(kp.SEL + (size_t)b * L * DS, (long)(k.t_last + 1) * (DS * 2));
    return k;
}

// Copy of tile tc into stage `sd` (LDS address of stage 0 = lds0).  A tile past the item's last one lies past the
// end of the raw segment: its copy moves zeros.
__device__ __forceinline__ CopyCtl make_copy(const Blk &k, int tc, int sd, int wave, unsigned lds0)
{
    CopyCtl c;
    const bool is_rep = tc < k.n_rep_tiles;
    const Seg &ps = is_rep ? k.rep_pool : k.raw_pool, &ss = is_rep ? k.rep_sel : k.raw_sel;
    c.pool_rs = int4v{(int)ps.lo, (int)ps.hi, (int)ps.bytes, RSRC_WORD3};
    c.sel_rs = int4v{(int)ss.lo, (int)ss.hi, (int)ss.bytes, RSRC_WORD3};
    const unsigned row0 = (is_rep ? tc * BN : k.raw_lo_blk + (tc - k.n_rep_tiles) * BN) + 8 * wave;   // first entry of this wavefront's share
    c.soff_lo = row0 * (DP * 2);
    c.soff_hi = c.soff_lo + 4 * (DP * 2);
    c.soff_sel = row0 * (DS * 2);
    c.m0_pool = lds0 + sd * STAGE_BYTES + 8 * wave * RSB;
    c.m0_sel = lds0 + sd * STAGE_BYTES + SEL_OFF + 8 * wave * (DS * 2);
    return c;
}

// What iteration tl of the tile loop needs besides the data: the copy of tile tl+3, this lane's read addresses in
// the stages of the S^T chain (tile tl+1) and of the O^T update (tile tl), and how tile tl is treated.
struct Ctl {
    CopyCtl cc;
    lds_cptr kb, vp0;
    KSel ksel;
    float bias;             // base-2 logit bias of tile tl (representatives may carry one)
    int is_rep, full;       // tile tl, as masks (-1 / 0): a tile of representatives; every entry visible to every row of this wavefront
};
// The same, computed in small steps (STEP 0..8) so that the work can be dealt out over the free issue slots of
// the O^T update; `t` carries intermediate values from step to step.  The empty assembly statements pin each
// step's results to its place (the compiler would otherwise gather the steps where their last result is needed).
struct CtlTmp { int tc, rep_c; unsigned row0, chain_lds, pv_lds; unsigned p0, p1, p2, q0, q1, q2; };
#define LCA_PIN_S(x) asm volatile("" : "+s"(x))
#define LCA_PIN_V(x) asm volatile("" : "+v"(x))
// -1 if a < b, else 0 (|a - b| < 2^31), by scalar arithmetic: a comparison result turned into an integer would travel
// through a vector register.  Unsigned subtraction so that the compiler cannot turn it back into a comparison.
__device__ __forceinline__ int lt_mask(int a, int b) { return (int)((unsigned)a - (unsigned)b) >> 31; }
template <int STEP>
__device__ __forceinline__ void ctl_step(Ctl &c, CtlTmp &t, const Blk &k, const MlaParams &kp, int tl, int wave, unsigned lds0, int k_off,
                                         int ksel_off, int v_off)
{
    if constexpr (STEP == 0) {
        t.tc = tl + 3;
        t.rep_c = lt_mask(t.tc, k.n_rep_tiles);
        c.is_rep = lt_mask(tl, k.n_rep_tiles);
        LCA_PIN_S(t.rep_c); LCA_PIN_S(c.is_rep);
    } else if constexpr (STEP == 1) {
        t.p0 = t.rep_c ? k.rep_pool.lo : k.raw_pool.lo;
        t.p1 = t.rep_c ? k.rep_pool.hi : k.raw_pool.hi;
        t.p2 = t.rep_c ? k.rep_pool.bytes : k.raw_pool.bytes;
        LCA_PIN_S(t.p0); LCA_PIN_S(t.p1); LCA_PIN_S(t.p2);
    } else if constexpr (STEP == 2) {
        t.q0 = t.rep_c ? k.rep_sel.lo : k.raw_sel.lo;
        t.q1 = t.rep_c ? k.rep_sel.hi : k.raw_sel.hi;
        t.q2 = t.rep_c ? k.rep_sel.bytes : k.raw_sel.bytes;
        LCA_PIN_S(t.q0); LCA_PIN_S(t.q1); LCA_PIN_S(t.q2);
    } else if constexpr (STEP == 3) {
        t.row0 = (t.rep_c ? t.tc * BN : k.raw_lo_blk + (t.tc - k.n_rep_tiles) * BN) + 8 * wave;
        LCA_PIN_S(t.row0);
    } else if constexpr (STEP == 4) {
        c.cc.soff_lo = t.row0 * (DP * 2);
        c.cc.soff_hi = c.cc.soff_lo + 4 * (DP * 2);
        c.cc.soff_sel = t.row0 * (DS * 2);
        LCA_PIN_S(c.cc.soff_lo); LCA_PIN_S(c.cc.soff_hi); LCA_PIN_S(c.cc.soff_sel);
    } else if constexpr (STEP == 5) {
        const unsigned sbase = lds0 + ((tl + 3) & (NSTAGE - 1)) * STAGE_BYTES;
        c.cc.m0_pool = sbase + 8 * wave * RSB;
        c.cc.m0_sel = sbase + SEL_OFF + 8 * wave * (DS * 2);
        LCA_PIN_S(c.cc.m0_pool); LCA_PIN_S(c.cc.m0_sel);
    } else if constexpr (STEP == 6) {
        // past the last tile the chain runs over a stage that holds zeros or an old tile: S^T that nobody reads
        t.chain_lds = lds0 + ((tl + 1) & (NSTAGE - 1)) * STAGE_BYTES;
        t.pv_lds = lds0 + (tl & (NSTAGE - 1)) * STAGE_BYTES;
        LCA_PIN_S(t.chain_lds); LCA_PIN_S(t.pv_lds);
    } else if constexpr (STEP == 7) {
        c.full = lt_mask(tl, k.rep_full_end) | (~lt_mask(tl, k.raw_full_lo) & lt_mask(tl, k.raw_full_hi));
        LCA_PIN_S(c.full);
        c.cc.pool_rs = int4v{(int)t.p0, (int)t.p1, (int)t.p2, RSRC_WORD3};
        c.cc.sel_rs = int4v{(int)t.q0, (int)t.q1, (int)t.q2, RSRC_WORD3};
    } else {
        unsigned kb = t.chain_lds + k_off, vp0 = t.pv_lds + v_off;
        c.ksel = make_ksel(t.chain_lds + ksel_off);
        c.bias = c.is_rep ? kp.bias_log2 : 0.f;
        LCA_PIN_V(kb); LCA_PIN_V(vp0); LCA_PIN_V(c.bias);
        LCA_PIN_V(c.ksel.a[0]); LCA_PIN_V(c.ksel.a[1]); LCA_PIN_V(c.ksel.a[2]); LCA_PIN_V(c.ksel.a[3]);
        c.kb = (lds_cptr)(uintptr_t)kb; c.vp0 = (lds_cptr)(uintptr_t)vp0;
    }
}
__device__ __forceinline__ Ctl make_ctl(const Blk &k, const MlaParams &kp, int tl, int wave, unsigned lds0, int k_off, int ksel_off, int v_off)
{
    Ctl c;
    CtlTmp t;
    ctl_step<0>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off); ctl_step<1>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off);
    ctl_step<2>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off); ctl_step<3>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off);
    ctl_step<4>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off); ctl_step<5>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off);
    ctl_step<6>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off); ctl_step<7>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off);
    ctl_step<8>(c, t, k, kp, tl, wave, lds0, k_off, ksel_off, v_off);
    return c;
}

// copies of tiles 0..2 of a work item into stages 0..2
__device__ __forceinline__ void issue_first_copies(const Blk &k, int wave, unsigned lds0, unsigned voff_pool, unsigned voff_sel)
{
    for (int tl = 0; tl < 3; ++tl) {
        const CopyCtl c = make_copy(k, tl, tl, wave, lds0);
        issue_copy_from<0>(c, voff_pool, voff_sel);
    }
}

// Queries of a work item.  The second product wants lane (n, G) to hold Q[row n][16 ks + 8 G .. +7] for every
// k-step ks, but loading them that way makes every load instruction touch 32 rows = 32 cache lines for 16 bytes
// each.  So the loads are issued row-wise -- load i = 4c + q: lane l fetches the 16-byte piece l%8 of the 128-byte
// column block c of row 8q + l/8, eight whole cache lines per instruction -- and q_to_fragments turns the
// registers into fragments through a private 4 KB LDS buffer, one column block (four k-steps) at a time.
__device__ __forceinline__ void load_q(const MlaParams &kp, const Blk &k, int wave, int lane, bf16x8 (&qf)[NKS])
{
    const int t_wfirst = k.t0 + wave * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int t = min(t_wfirst + 8 * q + (lane >> 3), kp.L - 1);
        const uint16_t *qp = kp.Q + (((size_t)k.b * kp.L + t) * kp.H + k.h) * DQK + (lane & 7) * 8;
#pragma unroll
        for (int c = 0; c < NKS / 4; ++c) qf[4 * c + q] = *reinterpret_cast<const bf16x8 *>(qp + c * 64);
    }
}
// `buf`: 4 KB of LDS private to this wavefront.  Piece p of row r sits at r*128 + ((p ^ (r>>1)) & 7)*16, which makes
// the row-wise writes and the fragment reads (16 lanes = 16 rows, one piece each) free of bank conflicts.  LDS
// operations of one wavefront run in order, so the reads of one block need no wait before the next block's writes.
__device__ __forceinline__ void q_to_fragments(char *buf, int lane, bf16x8 (&qf)[NKS])
{
    const int n = lane & 31, G = lane >> 5, wrow = lane >> 3, wp = lane & 7;
#pragma unroll
    for (int c = 0; c < NKS / 4; ++c) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = 8 * q + wrow;
            *reinterpret_cast<bf16x8 *>(buf + r * 128 + ((wp ^ (r >> 1)) & 7) * 16) = qf[4 * c + q];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) qf[4 * c + j] = *reinterpret_cast<const bf16x8 *>(buf + n * 128 + (((2 * j + G) ^ (n >> 1)) & 7) * 16);
    }
}

// Hide the entries of a boundary tile that this lane's query row must not see (e0 = first entry of the tile).
// Accumulator register r of lane group G holds entry e0 + acc_entry(r, 0) + G; a row sees the representatives
// [0, mt_row) or the raw tokens [raw_lo_row, t_row]: one unsigned comparison per register, no branches.
__device__ __forceinline__ void mask_tile(floatx16 &sv, const Blk &k, bool is_rep, int e0, int G)
{
    const int lo = is_rep ? -(1 << 30) : k.raw_lo_row, end = is_rep ? k.mt_row : k.t_row + 1;
    const unsigned count = (unsigned)(end - lo);         // may be 0: a row whose last token closes a group sees no raw token when w = 0
    const int d = e0 + G - lo;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        static_assert(acc_entry(5, 1) == acc_entry(5, 0) + 1, "lane group adds one to the entry");
        const bool vis = (unsigned)(d + acc_entry(r, 0)) < count;
        sv[r] = vis ? sv[r] : -INFINITY;
    }
}
// Largest base-2 logit of this lane's query row in one tile (both lanes of the row get it); -1e30 if it sees nothing.
// (inline assembly: the compiler would first canonicalise every input of a maximum it cannot see the origin of)
__device__ __forceinline__ float row_max(const floatx16 &sv, float c, float bias)
{
    float mx[6];
#pragma unroll
    for (int i = 0; i < 5; ++i) asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[i]) : "v"(sv[3 * i]), "v"(sv[3 * i + 1]), "v"(sv[3 * i + 2]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[5]) : "v"(mx[0]), "v"(mx[1]), "v"(mx[2]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[0]) : "v"(mx[3]), "v"(mx[4]), "v"(sv[15]));
    asm("v_max_f32 %0, %1, %2" : "=v"(mx[1]) : "v"(mx[5]), "v"(mx[0]));
    const float t = fmaxf(fmaf(mx[1], c, bias), NEG_BIG);
    // the partner lane holds the other 16 keys of this query: swap halves between two copies, no LDS traffic
    typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
    const uintx2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    float m;
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(sw[0]), "v"(sw[1]));
    return m;
}


// Persistent kernel: one workgroup per CU walks a list of work items.  Workgroup w lives on XCD w%8 (round-
// robin placement) and is slot w/8 of that XCD; the XCD's item list is (query blocks 2x, 2x+1, 2x+16, 2x+17, ...
// of the heaviest-first order) x (all heads), so that at any time the slots of an XCD work on the heads of two
// neighbouring query blocks, which see nearly the same keys, and share their K/V tiles in that XCD's L2.  The next item's queries and first
// tiles are requested before the current item's output is written, so the transition costs no round trip.
//
// Iteration tl of the tile loop, after its barrier: the held-back last MFMAs of the O^T update of tile tl-1
// (while the first key fragments of tile tl+1 arrive), the S^T chain of tile tl+1 with the softmax of tile tl
// in its shadow and the copy of tile tl+3 in its last slots, then the O^T update of tile tl with the loop's
// bookkeeping for iteration tl+1 in its shadow.
// UP variant, after the last tile: the head's value up-projection (section 3, Eq. 5: o = (sum_i p_i c_i) W^UV, the matrix
// the absorbed form leaves to the output side) applied to this wavefront's 32 rows while O^T is still in registers:
//   U^T[u, query] = sum_dv W[u, dv] O^T[dv, query]      A = W (4 tiles of 32 output dimensions, from memory), B = O^T
// Registers 8 hh .. 8 hh + 7 of accumulator tile i of lane group G are the rows dv = 32 i + 16 hh + {0..3, 8..11} + 4 G:
// normalised and rounded to the element type they ARE a B fragment of a 32x32x16 product whose k-slot (G, j) stands for
// that dv, so the A fragment of lane (u, G) is W[u][the same eight dv] -- two 8-byte pieces 16 bytes apart -- and
// nothing moves between lanes.  The output rounds O once to the element type before the product, as a separate
// projection of the stored O would.
template <bool F16>
__device__ __forceinline__ void up_project(const floatx16 (&acc)[NDV], float inv, const uint16_t *Wp_h, int lane, floatx16 (&up)[DU / 32])
{
    // Wp_h: this head's matrix in fragment order (pack_up_kernel): fragment (k-step, output tile) is 1 KB, lane l's 16 bytes at 16 l
    const char *wl = reinterpret_cast<const char *>(Wp_h) + lane * 16;
    constexpr int NF = 2 * NDV * (DU / 32), AHEAD = 8;     // 128 fragments, this many requested ahead of their use
    bf16x8 wf[AHEAD];
#pragma unroll
    for (int f = 0; f < AHEAD; ++f) wf[f] = *reinterpret_cast<const bf16x8 *>(wl + f * 1024);
#pragma unroll
    for (int mt = 0; mt < DU / 32; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) up[mt][r] = 0.f;
#pragma unroll
    for (int i = 0; i < NDV; ++i) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            union { bf16x8 v; bf16x2 b[4]; f16x2 h[4]; } of;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float x0 = acc[i][8 * hh + 2 * j] * inv, x1 = acc[i][8 * hh + 2 * j + 1] * inv;
                if (F16) of.h[j] = f16x2{(_Float16)x0, (_Float16)x1};
                else of.b[j] = bf16x2{(__bf16)x0, (__bf16)x1};
            }
#pragma unroll
            for (int mt = 0; mt < DU / 32; ++mt) {
                const int f = (2 * i + hh) * (DU / 32) + mt;
                up[mt] = pv_mfma<F16>(wf[f % AHEAD], of.v, up[mt]);
                if (f + AHEAD < NF) wf[f % AHEAD] = *reinterpret_cast<const bf16x8 *>(wl + (f + AHEAD) * 1024);
            }
            LCA_FENCE();
        }
    }
}

// W^UV of every head, [H, DU, DV] (output dimension major), into fragment order: for head h, k-step s = 2 i + hh and output
// tile mt, lane (u = l & 31, G = l >> 5) gets W[h][32 mt + u][32 i + 16 hh + {0..3, 8..11} + 4 G] as its 16 bytes.
__global__ __launch_bounds__(256) void pack_up_kernel(const uint16_t *__restrict__ W, uint16_t *__restrict__ Wp, int H)
{
    const int lane = threadIdx.x & 63;
    const long frag = (long)blockIdx.x * 4 + (threadIdx.x >> 6);       // over (h, k-step, output tile)
    if (frag >= (long)H * 2 * NDV * (DU / 32)) return;
    const int mt = frag % (DU / 32), s = (frag / (DU / 32)) % (2 * NDV), h = frag / ((DU / 32) * 2 * NDV);
    const uint16_t *src = W + ((size_t)h * DU + 32 * mt + (lane & 31)) * DV + 16 * s + 4 * (lane >> 5);
    uint2 lo = *reinterpret_cast<const uint2 *>(src), hi = *reinterpret_cast<const uint2 *>(src + 8);
    *reinterpret_cast<uint4 *>(Wp + (size_t)frag * 512 + lane * 8) = make_uint4(lo.x, lo.y, hi.x, hi.y);
}

template <bool F16, bool UP>
__global__ __launch_bounds__(256) void attn_mla_kernel(const MlaParams kp)
{
    __shared__ __attribute__((aligned(1024))) char stages[NSTAGE][STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, G = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = kp.L, H = kp.H;
    const unsigned lds0 = lds_address(&stages[0][0]);

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, n_slots = gridDim.x >> 3;
    const int n_units = kp.n_qb * kp.B;                       // (query block, sequence) pairs, heaviest first
    const int items_per_xcd = ((n_units + 15) / 16) * 2 * H;  // some may fall past n_units
    auto item = [&](int kidx, int &b, int &h, int &qb) {      // false when the item does not exist
        h = kidx % H;
        const int j = kidx / H, ord = (j >> 1) * 16 + 2 * xcd + (j & 1);     // an XCD works on two neighbouring query blocks at a time
        b = ord % kp.B;
        qb = kp.n_qb - 1 - ord / kp.B;
        return kidx < items_per_xcd && ord < n_units;
    };

    // per-lane LDS byte offsets
    const int krow = lds_row_of_m(n);                                                // LDS row behind S^T row n
    const int k_off = krow * RSB + G * 16;                                           // S^T, latent part: 16-byte chunk G of that row
    const int xs = (krow >> 1) & 7;                                                  // swizzle of that row in the RoPE part
    const int ksel_off = SEL_OFF + krow * (DS * 2) + (((G ^ xs) & 7) << 4);          // S^T, RoPE part: chunk (2j+G) sits at slot (2j+G)^xs; this is j = 0
    const int v_off = (4 * ((lane & 15) >> 2) + G) * RSB + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;   // V^T transpose read
    // copy side: lane l of a latent-row copy moves chunk l; lane l of the RoPE copy fills slot l&7 of local row l>>3
    // (row 8*wave + (l>>3) of the tile) with the chunk the swizzle assigns to that slot
    const unsigned voff_pool = lane * 16;
    const unsigned voff_sel = (lane >> 3) * (DS * 2) + (((lane & 7) ^ ((4 * wave + (lane >> 4)) & 7)) << 4);
    const float c = kp.scale_log2;

    int kidx = slot, ib, ih, iqb;
    while (kidx < items_per_xcd && !item(kidx, ib, ih, iqb)) kidx += n_slots;   // items past n_units only sit at the list's end
    if (kidx >= items_per_xcd) return;
    Blk cur = make_blk(kp, ib, ih, iqb, wave, n);

    bf16x8 qf[NKS];
    floatx16 acc[NDV];
    RowState st;
    issue_first_copies(cur, wave, lds0, voff_pool, voff_sel);
    load_q(kp, cur, wave, lane, qf);
    char *const qbuf = &stages[3][0] + wave * 32 * (128 * 2 + 16);      // this wavefront's part of the output staging area
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    q_to_fragments(qbuf, lane, qf);

    while (true) {
        // Pass 0 is the normal one: every row fixes its reference at the first entries it sees and never looks at
        // maxima again.  Only if a row sum ends beyond L_LIMIT (or not finite) the workgroup finds every row's true
        // maximum (S^T chains alone) and runs the item again from those (pass 2).
        int pass = 0;
        float m_exact = NEG_BIG;
        while (true) {       // passes over this item
        // O^T = 0: sixteen MFMAs with zero operands instead of 256 register writes (the matrix core is idle here anyway)
        {
            bf16x8 zf = {0, 0, 0, 0, 0, 0, 0, 0};
            asm volatile("" : "+v"(zf));
#pragma unroll
            for (int i = 0; i < NDV; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc[i]) : "v"(zf));   // (zeros in either type)
        }
        st.m_ref = m_exact; st.l_run = 0.f; st.p_max = 0.f;
        bool need_ref = pass == 0;          // wave-uniform: some row of this wavefront has no reference yet

        // the first tiles and the queries of this item are on their way; then the S^T chain of tile 0
        floatx16 snext, scur;
        Pb pb;
        PvFrags pvf;
        ChainFrags cf;
        // there is no tile -1: its held-back MFMAs add V^T = 0 times P^T = 0
#pragma unroll
        for (int i = 0; i < PV_GROUP; ++i) { pvf.lo[1][i] = bf16x4{0, 0, 0, 0}; pvf.hi[1][i] = bf16x4{0, 0, 0, 0}; }
        pb.v[0] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0}; pb.v[1] = pb.v[0];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        {
            lds_cptr s0 = (lds_cptr)(uintptr_t)lds0;
            const KSel ks0 = make_ksel(lds0 + ksel_off);
            chain_prefetch(cf, s0 + k_off, ks0);
            chain_and_softmax<false, false, F16>(cf, s0 + k_off, ks0, qf, snext, snext, pb, st, c, 0.f, pvf, s0, CopyCtl(), 0, 0);
        }
        scur = snext;
        int tl0 = 0;
        asm volatile("" : "+s"(tl0));        // (opaque: with a known zero the compiler turns the flag arithmetic of make_ctl back into comparisons)
        Ctl ctl = make_ctl(cur, kp, tl0, wave, lds0, k_off, ksel_off, v_off);

        for (int tl = 0; tl < cur.n_tiles; ++tl) {
            if (__builtin_expect((ctl.full == 0) | need_ref, 0)) {      // rare: boundary tiles, and the first tiles of an item
                if (ctl.full == 0) mask_tile(scur, cur, ctl.is_rep != 0, ctl.is_rep ? tl * BN : cur.raw_lo_blk + (tl - cur.n_rep_tiles) * BN, G);
                if (need_ref) {              // the first visible entries of a row fix its reference
                    const float mx = row_max(scur, c, ctl.bias);
                    st.m_ref = (st.m_ref == NEG_BIG) ? (F16 ? mx + REF_SHIFT_F16 : mx) : st.m_ref;    // (-1e30 + 4 is -1e30)
                    need_ref = __builtin_amdgcn_ballot_w64(st.m_ref == NEG_BIG) != 0;
                }
            }
            // tile tl+1 has landed: its copy was issued two iterations ago, only tile tl+2's 9 loads may be pending ...
            // and this wavefront's transpose reads of tile tl-1 (the held-back group) are in registers
            asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory");
            __syncthreads();      // ... for every wavefront, and every wavefront is done with tile tl-1 (all of its V^T fragments are in registers)
            LCA_FENCE();
            chain_prefetch(cf, ctl.kb, ctl.ksel);
            pv_tail<F16>(pvf, pb, acc);
            chain_and_softmax<true, true, F16>(cf,
                                          ctl.kb, ctl.ksel, qf, snext, scur, pb, st, c, ctl.bias, pvf, ctl.vp0, ctl.cc, voff_pool, voff_sel);
            Ctl nx;
            CtlTmp tmp;
            pv_update<F16>(pvf, ctl.vp0, pb, acc, [&](int j) {
                // Nothing may read the chain's result before MFMAs of the O^T update have run (the compiler takes an
                // inline-assembly result as ready at once; these MFMAs are the wait states it actually needs).
                if (j >= 4 && j < 20) asm volatile("v_mov_b32 %0, %1" : "=v"(scur[j - 4]) : "v"(snext[j - 4]));
                // the bookkeeping of iteration tl+1, a few instructions per MFMA
                switch (j) {
                case 1: ctl_step<0>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 3: ctl_step<1>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 5: ctl_step<2>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 7: ctl_step<3>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 9: ctl_step<4>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 11: ctl_step<5>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 13: ctl_step<6>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 15: ctl_step<7>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                case 21: ctl_step<8>(nx, tmp, cur, kp, tl + 1, wave, lds0, k_off, ksel_off, v_off); break;
                default: break;
                }
            });
            ctl = nx;
        }
        pv_tail<F16>(pvf, pb, acc);                        // the last tile's held-back MFMAs
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the trailing copies have landed before the stages are reused
        // every wavefront is done with the tile stages; repeat the item if a row sum ran out of range
        {
            const float l_chk = st.l_run + __shfl_xor(st.l_run, 32, 64);
            const bool redo = pass == 0 && (!(l_chk <= L_LIMIT) | (F16 && st.p_max > P_LIMIT_F16));
            if (!__syncthreads_or(redo)) break;
            {
                // exact row maxima, one tile at a time (no overlap: this path is rare): tile tl goes into stage tl%2
                // after the barrier of tile tl-1, which every wavefront reaches after its chain over tile tl-2
                m_exact = NEG_BIG;
                for (int tl = 0; tl < cur.n_tiles; ++tl) {
                    const CopyCtl cc = make_copy(cur, tl, tl & 1, wave, lds0);
                    issue_copy_from<0>(cc, voff_pool, voff_sel);
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    __syncthreads();
                    lds_cptr sp = (lds_cptr)(uintptr_t)(lds0 + (tl & 1) * STAGE_BYTES);
                    floatx16 sv;
                    ChainFrags cf;
                    PvFrags unused;
                    const KSel ksp = make_ksel(lds0 + (tl & 1) * STAGE_BYTES + ksel_off);
                    chain_prefetch(cf, sp + k_off, ksp);
                    chain_and_softmax<false, false, F16>(cf, sp + k_off, ksp, qf, sv, sv, pb, st, c, 0.f, unused, sp, CopyCtl(), 0, 0);
                    const bool is_rep = tl < cur.n_rep_tiles;
                    mask_tile(sv, cur, is_rep, is_rep ? tl * BN : cur.raw_lo_blk + (tl - cur.n_rep_tiles) * BN, G);
                    m_exact = fmaxf(m_exact, row_max(sv, c, is_rep ? kp.bias_log2 : 0.f));
                }
                __syncthreads();
                pass = 2;
                issue_first_copies(cur, wave, lds0, voff_pool, voff_sel);
            }
        }
        }

        // request the next item's first tiles (stages 0..2) and queries before writing this item's output
        int nb, nh, nqb;
        kidx += n_slots;
        const bool has_next = item(kidx, nb, nh, nqb);
        const int out_b = cur.b, out_h = cur.h, out_t0 = cur.t0;
        const float l_tot = st.l_run + __shfl_xor(st.l_run, 32, 64);
        const float inv = 1.f / l_tot;
        floatx16 up[UP ? DU / 32 : 1];
        // The lane number is taken afresh for everything from here on.  Values derived from it before the loop are kept in
        // spilled registers, and every reload from scratch memory is a round trip of its own that also waits for ALL
        // vector-memory operations in flight: below, the next item's queries and first tiles and the output stores.
        const int lane_here = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        const int n_here = lane_here & 31, G_here = lane_here >> 5;
        if (has_next) {
            cur = make_blk(kp, nb, nh, nqb, wave, n_here);
            // The queries first: behind the copies, anything their addresses still need from scratch memory would wait
            // for the tiles to arrive from HBM before the first query load could even be issued.
            if (!UP) load_q(kp, cur, wave, lane_here, qf);
            issue_first_copies(cur, wave, lds0, lane_here * 16,
                               (lane_here >> 3) * (DS * 2) + (((lane_here & 7) ^ ((4 * wave + (lane_here >> 4)) & 7)) << 4));
        }
        if constexpr (UP) {
            // (the projection needs the registers the next item's queries would take: those are requested after it)
            up_project<F16>(acc, inv, kp.W_up + (size_t)out_h * DU * DV, lane, up);
            if (has_next) load_q(kp, cur, wave, lane_here, qf);
        }

        // ---- epilogue: normalise, transpose through LDS stage 3 (four passes of 128 value columns), store coalesced ----
        constexpr int ORS = 128 * 2 + 16;                    // staging row stride (bytes)
        static_assert(4 * 32 * ORS <= STAGE_BYTES, "output staging must fit in one tile stage");
        char *obuf = &stages[3][0] + wave * 32 * ORS;
        const int t_wfirst = out_t0 + wave * 32;
        // The stores go through a buffer descriptor of this wavefront's rows of this head (row r at r*H*1 KB): scalar
        // offsets instead of 64-bit address arithmetic per store, and rows past the end of the sequence fall outside
        // the descriptor's range and are dropped.
        const int rows_valid = min(max(L - t_wfirst, 0), 32);
        constexpr int DO = UP ? DU : DV;                     // width of an output row
        const __amdgpu_buffer_rsrc_t o_rs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(kp.O + (((size_t)out_b * L + t_wfirst) * H + out_h) * DO), (short)0,
            rows_valid > 0 ? ((rows_valid - 1) * H * DO + DO) * 2 : 0, RSRC_WORD3);
        const int o_voff = ((lane_here >> 4) * H * DO + (lane_here & 15) * 8) * 2;
#pragma unroll
        for (int pass = 0; pass < DO / 128; ++pass) {
#pragma unroll
            for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    union { bf16x4 h; f16x4 hf; uint2 u; } o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float x = UP ? up[d4][r4 * 4 + i] : acc[pass * 4 + d4][r4 * 4 + i] * inv;
                        if (F16) o.hf[i] = (_Float16)x;
                        else o.h[i] = (__bf16)x;
                    }
                    *reinterpret_cast<uint2 *>(obuf + n_here * ORS + (d4 * 32 + 8 * r4 + 4 * G_here) * 2) = o.u;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r4 = 0; r4 < 8; ++r4) {                 // one wave-wide store covers four rows of 256 B
                typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
                const int r = r4 * 4 + (lane_here >> 4);
                const uintx4 v = *reinterpret_cast<const uintx4 *>(obuf + r * ORS + (lane_here & 15) * 16);
                __builtin_amdgcn_raw_buffer_store_b128(v, o_rs, o_voff, (r4 * 4 * H * DO + pass * 128) * 2, 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (kp.lse != nullptr) {
            const int t_row_here = t_wfirst + n_here;
            if (G_here == 0 && t_row_here < L)
                kp.lse[((size_t)out_b * L + t_row_here) * H + out_h] = (st.m_ref + log2f(l_tot)) * 0.6931471805599453f;
        }
        if (!has_next) break;
        // the next item's queries have been on their way since before the output was written; the wait leaves the output
        // stores (and, when they were issued after the queries, the first tiles' copies) in flight: vector-memory operations
        // complete in the order issued
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DO / 128) * 8 + (UP ? 0 : 3 * COPIES_PER_TILE)) : "memory");
        // (the fresh lane number again: the eight LDS addresses q_to_fragments derives from it would otherwise be kept across
        // the whole item, in spilled registers)
        q_to_fragments(qbuf, lane_here, qf);
    }
}

}  // namespace

bool attn_mla_supported(const Dims &d)
{
    // segment sizes and row offsets travel as 32-bit byte counts
    return (d.dtype == LCA_BF16 || d.dtype == LCA_F16) && d.mode == LCA_MODE_MLA && d.d_pool == DP && d.d_sel == DS && d.scale > 0.f && d.L <= (1 << 21);
}

size_t attn_mla_up_workspace_bytes(const Dims &d) { return attn_mla_supported(d) ? (size_t)d.H * DU * DV * 2 : 0; }

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
    const long items = (((long)kp.n_qb * d.B + 15) / 16) * 16 * d.H;
    const long cus = persistent_grid();
    long grid = items < cus ? items : cus;
    grid = (grid + 7) / 8 * 8;
    kp.W_up = nullptr;
    if (a.W_up != nullptr) {
        // the matrices in fragment order, in the caller's workspace (2 MB for 16 heads; microseconds)
        const long frags = (long)d.H * 2 * NDV * (DU / 32);
        pack_up_kernel<<<(unsigned)((frags + 3) / 4), 256, 0, st>>>((const uint16_t *)a.W_up, (uint16_t *)a.up_scratch, d.H);
        kp.W_up = (const uint16_t *)a.up_scratch;
        if (d.dtype == LCA_F16) attn_mla_kernel<true, true><<<(unsigned)grid, 256, 0, st>>>(kp);
        else attn_mla_kernel<false, true><<<(unsigned)grid, 256, 0, st>>>(kp);
    } else {
        if (d.dtype == LCA_F16) attn_mla_kernel<true, false><<<(unsigned)grid, 256, 0, st>>>(kp);
        else attn_mla_kernel<false, false><<<(unsigned)grid, 256, 0, st>>>(kp);
    }
    return hipGetLastError();
}

}  // namespace lca
