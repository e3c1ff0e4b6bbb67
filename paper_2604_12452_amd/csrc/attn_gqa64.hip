// bf16 / fp16 MFMA attention kernel for the GQA widths (d_k = d_v = 128), any number of query heads per KV
// head, on gfx950: prefill over the condensed context with hard-selected keys and pooled values per KV head
// (section 5.4 of the paper; attention as in section 4.3, Eq. 10 with the per-query partition of appendix
// A.2) and, with dense = 1, plain causal attention (section 3, Eq. 5).
//
// One wavefront per SIMD, as in the MLA kernel: with a single wavefront every instruction costs about five
// cycles of issue and an MFMA occupies the matrix core for 32, so the loop is laid out as one MFMA followed by
// a fixed, small number of other instructions.  At d = 128 a block of 32 x 32 (query, key) pairs costs 16 MFMAs
// and 16 exponentials per lane (56 vector instructions), 3.5 per MFMA before any operand is read, so operands
// must be cheap: a wavefront owns 64 query rows of ONE query head (two blocks of 32), and every key fragment and
// every value fragment it reads from LDS feeds two MFMAs.
//
// Workgroup = 4 wavefronts = the four query heads of one KV head (of one group of four) x the same 64 query rows:
// they see exactly the same keys and share every key/value tile.  (With 2 or 1 heads per KV head the wavefronts
// are 2 heads x 2 groups of 64 rows, or 4 groups of 64 rows of one head.)  Tiles of 64 entries (K and V rows of 256 B)
// are copied by direct-to-LDS loads into four 32 KB stages, three tiles ahead.  Rows sit at a 256-byte stride
// with their 16-byte chunks XOR-swizzled by row (at the source address of the copy), which keeps both read
// patterns bank-conflict-free:
//   S^T[key, query] = K Q^T      16-byte key reads, lane = S^T row m reads LDS row pi(m)
//   O^T[dv, query] += V^T P^T    transpose reads (ds_read_b64_tr_b16), each 16-lane block touches rows 4 apart
// with pi(8h + 4G + j) = 4j + 2h + G inside each 16 rows (the S^T accumulator registers then already are the B
// fragments of the second product).
//
// Software pipeline over halves of 32 entries.  Slot H holds, in this order,
//     O^T update of half H-1   (16 MFMAs: 8 value fragments x 2 row blocks),
//     S^T chain of half H+1    (16 MFMAs: 8 key fragments x 2 row blocks),
// with the softmax of half H (32 exponentials per lane) dealt out one element per MFMA over all 32.  The key
// fragments of the chain are requested during the update, the value fragments of the next slot's update
// during the chain.  Iteration T = slot 2T, barrier, slot 2T+1: the chain of slot 2T+1 is the first to read tile
// T+1, and every wavefront is done with tile T-1 after slot 2T, so the barrier sits between the two and the
// 16 MFMAs of the update that follows it cover the arrival of the first key fragments.
//
// Softmax uses one fixed reference per row (the first entries the row sees), so O^T is never rescaled and no
// maxima are taken in the steady state; a row sum that ends beyond 2^90 makes the workgroup find exact maxima
// (S^T chains alone) and run the item again from those.
#include <type_traits>

#include "lca_internal.h"

namespace lca {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// fp16 runs through the same code (template parameter F16): fragments travel in the bf16 vector types as plain 16-bit
// containers, and only the matrix instructions, the two conversions (P^T, output) and the softmax range differ.
union Pb { bf16x8 v[2]; bf16x2 p[8]; };     // P^T of one half and row block: the B operands of the two k-steps of the second product

#define LCA_FENCE() __builtin_amdgcn_sched_barrier(0)
#define LCA_PIN_S(x) asm volatile("" : "+s"(x))
#define LCA_PIN_V(x) asm volatile("" : "+v"(x))

constexpr int D = 128;                  // d_k = d_v
constexpr int BN = 64;                  // entries per tile (two halves of 32)
constexpr int RB = D * 2;               // row bytes
constexpr int V_OFF = BN * RB;          // the value rows of a stage start here
constexpr int STAGE_BYTES = 2 * BN * RB;   // 32 768
constexpr int NSTAGE = 4;
constexpr int NW = 4;                   // wavefronts per workgroup
constexpr int BMW = 64;                 // query rows per wavefront
constexpr int NKS = D / 16;             // 8 k-steps of S^T
constexpr int NDV = D / 32;             // 4 value tiles
constexpr int COPIES = 2 * BN / NW / 4; // direct-to-LDS loads per wavefront and tile: 16 rows of K and of V, 4 rows each
constexpr int GRID = 256;               // most workgroups the persistent kernel is launched with (one per CU of the chip)
constexpr int RING = 4;                 // fragments in flight per operand
constexpr float NEG_BIG = -1.0e30f;
constexpr float L_LIMIT = 0x1p90f;      // a row sum beyond this (or not finite) makes the workgroup repeat the item from exact maxima
// fp16 ends at 65504: the fp16 kernels keep the largest exponential of each row (one v_max3 per pair) and repeat the item
// from exact maxima if it left the type's range.  The reference sits 4 binades above the first maximum a row sees
// (first entries at 2^-4): later logits may be 2^19 times larger before that happens, at the price of 4 of fp16's 24
// binades at the bottom.
constexpr float P_LIMIT_F16 = 65000.f;
constexpr float REF_SHIFT_F16 = 4.f;
constexpr int RSRC_WORD3 = 0x00020000;  // raw buffer of dwords, gfx9 layout

struct G64Params {
    const uint16_t *Q, *K, *V, *k_rep, *v_rep;
    uint16_t *O;
    float *lse;
    int B, L, H, S, g, w, m, dense;
    int hw, hgs;        // query heads per work item (4, 2 or 1, a divisor of H/S: the wavefronts are hw heads x 4/hw groups of 64 rows); head groups per KV head
    int n_qb, n_units;  // query blocks (of 256/hw rows) per sequence; KV-sharing units = B * S * hgs
    unsigned g_magic, units_magic, hgs_magic, s_magic;     // for divisions by g, n_units, hgs and S (udiv_small)
    float scale_log2, bias_log2;
};

// x / d for d >= 1 and x * d < 2^32, with magic = 2^32 / d + 1 (rounded down) from the host: one multiplication instead
// of the thirty-odd instructions of a 32-bit division (a work item is short enough for a dozen of those to show).
__device__ __forceinline__ unsigned udiv_small(unsigned x, unsigned d, unsigned magic) { return d == 1 ? x : __umulhi(x, magic); }

__device__ __forceinline__ constexpr int lds_row_of_m(int m) { return (m & 16) + 4 * (m & 3) + 2 * ((m >> 3) & 1) + ((m >> 2) & 1); }
__device__ __forceinline__ constexpr int acc_entry(int r, int G) { return lds_row_of_m(8 * (r >> 2) + 4 * G + (r & 3)); }
__device__ __forceinline__ unsigned lds_address(const void *p) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p; }
// -1 if a < b, else 0 (|a - b| < 2^31), by scalar arithmetic; unsigned so that the compiler cannot turn it back into a
// comparison (whose result, turned into an integer, would travel through a vector register)
__device__ __forceinline__ int lt_mask(int a, int b) { return (int)((unsigned)a - (unsigned)b) >> 31; }

// A segment of keys or values as the first three words of a raw buffer descriptor: rows past its end read as zeros.
struct Seg { unsigned lo, hi, bytes; };
__device__ __forceinline__ Seg make_seg(const void *p, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)p;
    return Seg{(unsigned)a, (unsigned)(a >> 32) & 0xFFFFu, bytes};
}

// One direct-to-LDS load of 64 x 16 bytes: lane l fetches segment bytes [soff + voff, +16) into LDS bytes
// [m0_base + M0_ADD + 16 l, +16).  Inline assembly: the compiler would make every later LDS read wait for a
// direct-to-LDS load it knows about; ordering is by hand (s_waitcnt vmcnt + workgroup barrier before a stage is read).
template <int M0_ADD>
__device__ __forceinline__ void dma_1k(unsigned voff, const int4v &rs, unsigned soff, unsigned m0_base)
{
    asm volatile("s_add_u32 m0, %2, %4\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %3 offen lds"
                 : : "v"(voff), "s"(rs), "s"(m0_base), "s"(soff), "n"(M0_ADD) : "scc", "memory");
}

// Everything one wavefront needs to know about one work item = 256/hw query rows of the hw heads of one head group.
struct Blk {
    int b, h, t0, t_last, t_w0;              // sequence, this wavefront's query head, first / last query row of the item, first of the wavefront
    int t_row[2], mt_row[2], raw_lo_row[2];  // per lane and row block: query row, representatives it sees, first raw token it sees
    int raw_lo_blk, mt_blk_hi;               // first raw token / representatives any row of the block sees
    int n_rep_tiles, n_tiles;
    int rep_full_end, raw_full_lo, raw_full_hi;   // tiles every row of this wavefront sees completely (no masking)
    Seg rep_k, rep_v, raw_k, raw_v;
    unsigned rep_stride, raw_stride;         // bytes between rows of a segment
};

__device__ __forceinline__ Blk make_blk(const G64Params &kp, int unit, int qb, int wave, int n)
{
    Blk k;
    const int L = kp.L, g = kp.g, w = kp.w, hps = kp.H / kp.S;
    auto groups_visible = [&](int t) { return (kp.dense || t + 1 <= w) ? 0 : (int)udiv_small(t + 1 - w, g, kp.g_magic); };
    const int uq = udiv_small(unit, kp.hgs, kp.hgs_magic), hg = unit - uq * kp.hgs;
    k.b = udiv_small(uq, kp.S, kp.s_magic);
    const int s = uq - k.b * kp.S;
    const int hi = wave & (kp.hw - 1), rg = wave / kp.hw, rows = BMW * (NW / kp.hw);     // hw is 1, 2 or 4
    k.h = s * hps + hg * kp.hw + hi;
    k.t0 = qb * rows;
    k.t_last = min(k.t0 + rows, L) - 1;
    k.t_w0 = k.t0 + rg * BMW;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        k.t_row[rb] = k.t_w0 + 32 * rb + n;
        k.mt_row[rb] = groups_visible(k.t_row[rb]);
        k.raw_lo_row[rb] = k.mt_row[rb] * g;
    }
    const int mt_w_lo = groups_visible(k.t_w0), mt_w_hi = groups_visible(k.t_w0 + BMW - 1);
    k.mt_blk_hi = groups_visible(k.t_last);
    k.raw_lo_blk = groups_visible(k.t0) * g;
    k.n_rep_tiles = (k.mt_blk_hi + BN - 1) / BN;
    k.n_tiles = k.n_rep_tiles + (k.t_last + 1 - k.raw_lo_blk + BN - 1) / BN;
    k.rep_full_end = mt_w_lo / BN;
    k.raw_full_lo = k.n_rep_tiles + (mt_w_hi * g - k.raw_lo_blk + BN - 1) / BN;
    k.raw_full_hi = k.n_rep_tiles + max(0, (k.t_w0 + 1 - k.raw_lo_blk) / BN);
    // segments: representatives [B,S,m,128] (row stride 256 B), raw tokens [B,L,S,128] (row stride S*256 B)
    k.rep_stride = RB;
    k.raw_stride = kp.S * RB;
    const size_t rep_off = ((size_t)k.b * kp.S + s) * kp.m * D, raw_off = ((size_t)k.b * L * kp.S + s) * D;
    k.rep_k = make_seg(kp.k_rep + rep_off, (unsigned)k.mt_blk_hi * RB);
    k.rep_v = make_seg(kp.v_rep + rep_off, (unsigned)k.mt_blk_hi * RB);
    k.raw_k = make_seg(kp.K + raw_off, (unsigned)k.t_last * k.raw_stride + RB);
    k.raw_v = make_seg(kp.V + raw_off, (unsigned)k.t_last * k.raw_stride + RB);
    return k;
}

// What a wavefront needs to copy its 16 rows of K and of V of one tile into one stage (all wavefront-uniform).  The
// wavefront's rows are 4*wave + 16q + (0..3), q = 0..3: one load per q and operand.
struct CopyCtl {
    int4v k_rs, v_rs;
    unsigned soff[4];           // byte offsets of the wavefront's rows 0, 16, 32, 48 (+ 4*wave) in the segment
    unsigned m0;                // LDS address of the wavefront's first K row in the stage
    unsigned stride;            // bytes between rows of the segment
};
__device__ __forceinline__ CopyCtl make_copy(const Blk &k, int tc, int sd, int wave, unsigned lds0)
{
    CopyCtl c;
    const int is_rep = lt_mask(tc, k.n_rep_tiles);
    const Seg &ks = is_rep ? k.rep_k : k.raw_k, &vs = is_rep ? k.rep_v : k.raw_v;
    c.k_rs = int4v{(int)ks.lo, (int)ks.hi, (int)ks.bytes, RSRC_WORD3};
    c.v_rs = int4v{(int)vs.lo, (int)vs.hi, (int)vs.bytes, RSRC_WORD3};
    c.stride = is_rep ? k.rep_stride : k.raw_stride;
    const unsigned row0 = (is_rep ? tc * BN : k.raw_lo_blk + (tc - k.n_rep_tiles) * BN) + 4 * wave;
    c.soff[0] = row0 * c.stride;
    c.soff[1] = c.soff[0] + 16 * c.stride;
    c.soff[2] = c.soff[1] + 16 * c.stride;
    c.soff[3] = c.soff[2] + 16 * c.stride;
    c.m0 = lds0 + sd * STAGE_BYTES + 4 * wave * RB;
    return c;
}
// make_copy in four steps (STEP 0..3) of a few scalar instructions each, so that the tile loop can deal them out over
// steps that have issue slots to spare; `sel` carries the descriptor words from step to step.  The empty assembly
// statements pin each step's results to its place.
struct CopySel { int is_rep; unsigned k0, k1, k2, v0, v1, v2; };
template <int STEP>
__device__ __forceinline__ void copy_step(CopyCtl &c, CopySel &t, const Blk &k, int tc, int wave, unsigned lds0)
{
    if constexpr (STEP == 0) {
        t.is_rep = lt_mask(tc, k.n_rep_tiles);
        t.k0 = t.is_rep ? k.rep_k.lo : k.raw_k.lo;
        t.k1 = t.is_rep ? k.rep_k.hi : k.raw_k.hi;
        t.k2 = t.is_rep ? k.rep_k.bytes : k.raw_k.bytes;
        LCA_PIN_S(t.is_rep); LCA_PIN_S(t.k0); LCA_PIN_S(t.k1); LCA_PIN_S(t.k2);
    } else if constexpr (STEP == 1) {
        t.v0 = t.is_rep ? k.rep_v.lo : k.raw_v.lo;
        t.v1 = t.is_rep ? k.rep_v.hi : k.raw_v.hi;
        t.v2 = t.is_rep ? k.rep_v.bytes : k.raw_v.bytes;
        c.stride = t.is_rep ? k.rep_stride : k.raw_stride;
        LCA_PIN_S(t.v0); LCA_PIN_S(t.v1); LCA_PIN_S(t.v2); LCA_PIN_S(c.stride);
    } else if constexpr (STEP == 2) {
        const unsigned row0 = (t.is_rep ? tc * BN : k.raw_lo_blk + (tc - k.n_rep_tiles) * BN) + 4 * wave;
        c.soff[0] = row0 * c.stride;
        c.m0 = lds0 + (tc & (NSTAGE - 1)) * STAGE_BYTES + 4 * wave * RB;
        LCA_PIN_S(c.soff[0]); LCA_PIN_S(c.m0);
    } else {
        const unsigned s16 = 16 * c.stride;
        c.soff[1] = c.soff[0] + s16;
        c.soff[2] = c.soff[1] + s16;
        c.soff[3] = c.soff[2] + s16;
        LCA_PIN_S(c.soff[1]); LCA_PIN_S(c.soff[2]); LCA_PIN_S(c.soff[3]);
        c.k_rs = int4v{(int)t.k0, (int)t.k1, (int)t.k2, RSRC_WORD3};
        c.v_rs = int4v{(int)t.v0, (int)t.v1, (int)t.v2, RSRC_WORD3};
    }
}
// Copy Q (0..3: K rows 16Q + 4*wave + 0..3; 4..7: the V rows).  Lane l fills slot l&15 of row l>>4 of those four with the
// chunk the swizzle assigns to that slot: K chunk ^ (row & 15), V chunk ^ (row & 12), and row & 15 = 4*wave + (l>>4)
// whatever Q is, so the lane's byte offset voff_k / voff_v = (l>>4)*stride + 16*chunk is the same for every copy of a tile.
template <int Q>
__device__ __forceinline__ void issue_copy_part(const CopyCtl &c, unsigned voff_k, unsigned voff_v)
{
    if constexpr (Q < 4) dma_1k<Q * 16 * RB>(voff_k, c.k_rs, c.soff[Q], c.m0);
    else dma_1k<V_OFF + (Q - 4) * 16 * RB>(voff_v, c.v_rs, c.soff[Q - 4], c.m0);
}
template <int Q = 0>
__device__ __forceinline__ void issue_copy_all(const CopyCtl &c, unsigned voff_k, unsigned voff_v)
{
    if constexpr (Q < COPIES) {
        issue_copy_part<Q>(c, voff_k, voff_v);
        issue_copy_all<Q + 1>(c, voff_k, voff_v);
    }
}
__device__ __forceinline__ void issue_copy_dyn(int q, const CopyCtl &c, unsigned voff_k, unsigned voff_v)
{
    switch (q) {      // q is a constant after unrolling
    case 0: issue_copy_part<0>(c, voff_k, voff_v); break;
    case 1: issue_copy_part<1>(c, voff_k, voff_v); break;
    case 2: issue_copy_part<2>(c, voff_k, voff_v); break;
    case 3: issue_copy_part<3>(c, voff_k, voff_v); break;
    case 4: issue_copy_part<4>(c, voff_k, voff_v); break;
    case 5: issue_copy_part<5>(c, voff_k, voff_v); break;
    case 6: issue_copy_part<6>(c, voff_k, voff_v); break;
    default: issue_copy_part<7>(c, voff_k, voff_v); break;
    }
}

// Hide the entries of a boundary half-tile that this lane's query row must not see (e0 = first entry of the half).
// Accumulator register r of lane group G holds entry e0 + acc_entry(r, 0) + G; a row sees the representatives
// [0, mt_row) or the raw tokens [raw_lo_row, t_row]: one unsigned comparison per register.
__device__ __forceinline__ void mask_half(floatx16 &sv, bool is_rep, int mt_row, int raw_lo_row, int t_row, int e0, int G)
{
    const int lo = is_rep ? -(1 << 30) : raw_lo_row, end = is_rep ? mt_row : t_row + 1;
    const unsigned count = (unsigned)(end - lo);         // may be 0
    const int d = e0 + G - lo;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const bool vis = (unsigned)(d + acc_entry(r, 0)) < count;
        sv[r] = vis ? sv[r] : -INFINITY;
    }
}
// Largest base-2 logit of this lane's query row in one half-tile (both lanes of the row get it); -1e30 if it sees nothing.
__device__ __forceinline__ float row_max(const floatx16 &sv, float c, float bias)
{
    float mx[6];
#pragma unroll
    for (int i = 0; i < 5; ++i) asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[i]) : "v"(sv[3 * i]), "v"(sv[3 * i + 1]), "v"(sv[3 * i + 2]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[5]) : "v"(mx[0]), "v"(mx[1]), "v"(mx[2]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx[0]) : "v"(mx[3]), "v"(mx[4]), "v"(sv[15]));
    asm("v_max_f32 %0, %1, %2" : "=v"(mx[1]) : "v"(mx[5]), "v"(mx[0]));
    const float t = fmaxf(fmaf(mx[1], c, bias), NEG_BIG);
    typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
    const uintx2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(t), __float_as_uint(t), false, false);
    float m;
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(sw[0]), "v"(sw[1]));
    return m;
}

typedef __attribute__((address_space(3))) bf16x4 *lds_b64_ptr;
typedef const __attribute__((address_space(3))) bf16x8 *lds_b128_ptr;

// Per-lane LDS addresses of the operand fragments in the stage they currently point to; halves and k-steps are
// immediate offsets.
struct Addr {
    unsigned k[NKS];        // S^T operand: chunk 2ks+G of row krow sits at slot (2ks+G)^(krow&15)
    unsigned v[NDV];        // V^T operand per value tile: chunk c of row r sits at slot c^(r&12)
};
__device__ __forceinline__ bf16x8 load_k(const Addr &a, int half, int ks) { return *(lds_b128_ptr)(uintptr_t)(a.k[ks] + half * 32 * RB); }
// V^T fragment i = (k-step kk = i / 4, value tile dvt = i % 4) of a half: two transpose reads of four keys each
__device__ __forceinline__ bf16x8 load_v(const Addr &a, int half, int i)
{
    const unsigned o = (half * 32 + (i / NDV) * 16) * RB;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(uintptr_t)(a.v[i % NDV] + o));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b64_ptr)(uintptr_t)(a.v[i % NDV] + o + 2 * RB));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// per-lane softmax state of the two query rows (base-2 logits)
struct RowState { float m_ref[2], l_run[2], p_max[2]; };      // p_max, fp16 only: the largest exponential of the row so far

// Queries of a work item: the loads are issued row-wise -- load i: lane l fetches the 16-byte piece l&15 of row
// 4i + (l>>4), four whole rows per instruction -- and q_to_fragments turns the registers into the fragments of the
// first product (lane (n, G) holds Q[row n][16 ks + 8 G .. +7] of each row block) through 8 KB of LDS private to
// the wavefront, one row block at a time.  Piece p of row r sits at r*256 + ((p ^ r) & 15)*16: no bank conflicts
// either way.  LDS operations of one wavefront run in order, so nothing has to wait in between.
// (through a buffer descriptor of the item's rows of this head: one scalar offset per load instead of 64-bit address
// arithmetic, rows past the end of the sequence read as zeros)
__device__ __forceinline__ void load_q(const G64Params &kp, const Blk &k, int lane, bf16x8 (&qf)[2][NKS])
{
    const int rows_valid = min(max(kp.L - k.t_w0, 0), BMW);
    const __amdgpu_buffer_rsrc_t q_rs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(kp.Q + (((size_t)k.b * kp.L + k.t_w0) * kp.H + k.h) * D), (short)0, rows_valid > 0 ? ((rows_valid - 1) * kp.H * D + D) * 2 : 0, RSRC_WORD3);
    const int voff = ((lane >> 4) * kp.H * D + (lane & 15) * 8) * 2;
#pragma unroll
    for (int i = 0; i < 2 * NKS; ++i) {
        const uintx4 v = __builtin_amdgcn_raw_buffer_load_b128(q_rs, voff, 4 * i * kp.H * D * 2, 0);
        qf[i / NKS][i % NKS] = __builtin_bit_cast(bf16x8, v);
    }
}
__device__ __forceinline__ void q_to_fragments(char *buf, int lane, bf16x8 (&qf)[2][NKS])
{
    const int n = lane & 31, G = lane >> 5;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int i = 0; i < NKS; ++i) {
            const int r = 4 * i + (lane >> 4);     // row inside the row block
            *reinterpret_cast<bf16x8 *>(buf + r * RB + (((lane & 15) ^ r) & 15) * 16) = qf[rb][i];
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[rb][ks] = *reinterpret_cast<const bf16x8 *>(buf + n * RB + (((2 * ks + G) ^ n) & 15) * 16);
    }
}

// Persistent kernel: one workgroup per CU walks a list of work items.  Workgroup w lives on XCD w%8 (round-robin
// placement) and is slot w/8 of that XCD.  Items are numbered (query block, heaviest first) x (unit = sequence x KV
// head x head group) and item i belongs to XCD i%8: with a multiple of eight units every unit keeps to one XCD, whose
// L2 then holds that KV head's representatives and the sliding raw window.
template <bool F16>
__global__ __launch_bounds__(64 * NW, 1) void attn_gqa64_kernel(const G64Params kp)
{
    __shared__ __attribute__((aligned(1024))) char stages[NSTAGE][STAGE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, G = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = kp.L, H = kp.H;
    const unsigned lds0 = lds_address(&stages[0][0]);
    const float c = kp.scale_log2;

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, n_slots = gridDim.x >> 3;
    const int n_items = kp.n_qb * kp.n_units;
    auto item = [&](int kidx, int &unit, int &qb) {           // item kidx of this XCD; false past the end
        const int i = kidx * 8 + xcd;
        const int iq = udiv_small(i, kp.n_units, kp.units_magic);
        unit = i - iq * kp.n_units;
        qb = kp.n_qb - 1 - iq;
        return i < n_items;
    };

    // fragment addresses relative to stage 0
    Addr adr;
    {
        const int krow = lds_row_of_m(n), xk = krow & 15;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) adr.k[ks] = lds0 + krow * RB + (((2 * ks + G) ^ xk) << 4);
        const int p = lane & 15, j = p >> 2, blk = (lane >> 4) & 1, pp = (p & 3) >> 1;
#pragma unroll
        for (int dvt = 0; dvt < NDV; ++dvt) {
            const int row = 4 * j + G;                         // + 2*hh + 16*kk + 32*half
            const int chunk = 4 * dvt + 2 * blk + pp;
            adr.v[dvt] = lds0 + V_OFF + row * RB + ((chunk ^ (4 * j)) << 4) + 8 * (p & 1);
        }
    }
    // copy side: lane l moves piece l&15 of local row l>>4 (rows of the representatives are 256 B apart, raw rows S*256)
    const unsigned chunk_k = (((lane & 15) ^ (4 * wave + (lane >> 4))) << 4), chunk_v = (((lane & 15) ^ (4 * wave)) << 4);

    int kidx = slot, iu, iqb;
    if (!item(kidx, iu, iqb)) return;
    Blk cur = make_blk(kp, iu, iqb, wave, n);

    bf16x8 qf[2][NKS];
    floatx16 acc[2][NDV];
    RowState st;
    char *const qbuf = &stages[3][0] + wave * (32 * RB);
    auto issue_first_copies = [&](const Blk &k) {
        for (int tl = 0; tl < 3; ++tl) {
            const CopyCtl cc = make_copy(k, tl, tl, wave, lds0);
            issue_copy_all(cc, (lane >> 4) * cc.stride + chunk_k, (lane >> 4) * cc.stride + chunk_v);
        }
    };
    issue_first_copies(cur);
    load_q(kp, cur, lane, qf);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    q_to_fragments(qbuf, lane, qf);

    while (true) {
        int pass = 0;
        float m_exact[2] = {NEG_BIG, NEG_BIG};
        while (true) {       // passes over this item: 0 = normal; 2 = again, from exact maxima
            // O^T = 0 by MFMAs with zero operands
            {
                bf16x8 zf = {0, 0, 0, 0, 0, 0, 0, 0};
                asm volatile("" : "+v"(zf));
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int i = 0; i < NDV; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(acc[rb][i]) : "v"(zf));
            }
            st.m_ref[0] = m_exact[0]; st.m_ref[1] = m_exact[1]; st.l_run[0] = 0.f; st.l_run[1] = 0.f; st.p_max[0] = 0.f; st.p_max[1] = 0.f;
            bool need_ref = pass == 0;

            floatx16 s[2][2];            // S^T of half H and row block rb lives in s[H % 2][rb]
            Pb pb[2][2];                 // P^T likewise
            bf16x8 kf[RING], vf[RING];
            float nb[2] = {0.f, 0.f};
            Addr a = adr;                // a.k: the stage of the tile whose keys the next chain reads; a.v: one tile behind from mid-iteration on
            auto next_stage = [&](int t) { return (t & (NSTAGE - 1)) == NSTAGE - 1 ? -(NSTAGE - 1) * STAGE_BYTES : STAGE_BYTES; };

            // Softmax of half `par`, element by element: element e = 0..31 is accumulator register 2*(e/4) + e%2 of row
            // block (e/2)%2, so that two consecutive elements are one bf16 pair of the second product's operand.  Step e
            // issues the exponential of element e and finishes element e-1 (its share of the row sum and, with every
            // second element, the rounding of the pair): an instruction that reads an exponential right behind it costs
            // a wait state, one step later it costs none.  The empty assembly statements pin the work to its place.
            float p_prev = 0.f, p_prev2 = 0.f;
            auto softmax_finish = [&](int par, int e) {        // element e, whose exponential is p_prev (and p_prev2 that of e-1)
                const int rb = (e >> 1) & 1;
                st.l_run[rb] += p_prev;
                LCA_PIN_V(st.l_run[rb]);
                if (e & 1) {
                    if (F16) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(st.p_max[rb]) : "v"(p_prev2), "v"(p_prev));
                    unsigned bits;
                    if (F16) bits = __builtin_bit_cast(unsigned, f16x2{(_Float16)p_prev2, (_Float16)p_prev});
                    else bits = __builtin_bit_cast(unsigned, bf16x2{(__bf16)p_prev2, (__bf16)p_prev});
                    LCA_PIN_V(bits);
                    pb[par][rb].p[(e >> 2)] = __builtin_bit_cast(bf16x2, bits);
                }
            };
            auto softmax_step = [&](int par, int e) {
                const int rb = (e >> 1) & 1, r = 2 * (e >> 2) + (e & 1);
                float p = __builtin_amdgcn_exp2f(fmaf(s[par][rb][r], c, nb[rb]));
                if (e > 0) softmax_finish(par, e - 1);
                LCA_PIN_V(p);           // the exponential belongs to this step too (pinned behind the other work: right behind the
                                        // exponential the statement would cost a wait state)
                p_prev2 = p_prev;
                p_prev = p;
            };
            // The softmax work that follows MFMA m = 0..31 of a slot: none after the first two (the chain that ended just
            // before the slot may still be writing the S^T registers), then one element per MFMA, two after the last two.
            auto softmax_after = [&](int par, int m) {
                if (m >= 2 && m < 30) softmax_step(par, m - 2);
                if (m == 30) { softmax_step(par, 28); softmax_step(par, 29); }
                if (m == 31) { softmax_step(par, 30); softmax_step(par, 31); softmax_finish(par, 31); }
            };
            // S^T chain step (k-step ks, row block rb) into s[par][rb]; assembly so that the accumulator is a vector
            // register tuple that the vector ALU can read as it is
            auto chain_mfma = [&](int par, int rb, int ks, const bf16x8 &kfrag) {
                if (F16) {
                    if (ks == 0) asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(s[par][rb]) : "v"(kfrag), "v"(qf[rb][ks]));
                    else asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(s[par][rb]) : "v"(kfrag), "v"(qf[rb][ks]));
                } else {
                    if (ks == 0) asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s[par][rb]) : "v"(kfrag), "v"(qf[rb][ks]));
                    else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s[par][rb]) : "v"(kfrag), "v"(qf[rb][ks]));
                }
            };

            // How tile tl is treated (wavefront-uniform): segment, first entry, whether nothing has to be masked
            struct TileInfo { int is_rep, full, e0; float bias; };
            auto tile_info = [&](int tl) {
                TileInfo ti;
                ti.is_rep = lt_mask(tl, cur.n_rep_tiles);
                ti.full = lt_mask(tl, cur.rep_full_end) | (~lt_mask(tl, cur.raw_full_lo) & lt_mask(tl, cur.raw_full_hi));
                ti.e0 = ti.is_rep ? tl * BN : cur.raw_lo_blk + (tl - cur.n_rep_tiles) * BN;
                ti.bias = ti.is_rep ? kp.bias_log2 : 0.f;
                return ti;
            };
            // Before the softmax of a half: masks of boundary tiles and, while a row has no reference yet, the reference
            // (the first visible entries fix it).  Rare; the wait states keep the vector ALU off S^T registers that the
            // last MFMA of the chain may still be writing.
            auto prepare_half = [&](int par, int half, const TileInfo &ti) {
                if (__builtin_expect((ti.full == 0) | need_ref, 0)) {
                    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        asm volatile("" : "+v"(s[par][rb]));
                        if (ti.full == 0) mask_half(s[par][rb], ti.is_rep != 0, cur.mt_row[rb], cur.raw_lo_row[rb], cur.t_row[rb], ti.e0 + 32 * half, G);
                        if (need_ref) {
                            const float mx = row_max(s[par][rb], c, ti.bias);
                            st.m_ref[rb] = (st.m_ref[rb] == NEG_BIG) ? (F16 ? mx + REF_SHIFT_F16 : mx) : st.m_ref[rb];    // (-1e30 + 4 is -1e30)
                        }
                    }
                    if (need_ref) need_ref = __builtin_amdgcn_ballot_w64((st.m_ref[0] == NEG_BIG) | (st.m_ref[1] == NEG_BIG)) != 0;
                }
                nb[0] = ti.bias - st.m_ref[0];
                nb[1] = ti.bias - st.m_ref[1];
            };

            // Slot H (par = H % 2): O^T update of half H-1 (its P^T is pb[1-par]; its V^T fragments are half `1-par` of the
            // tile a.v points to), softmax of half H (S^T in s[par]), S^T chain of half H+1 into s[1-par] (its keys are half
            // `1-par` of the tile a.k points to).  PV / SM switch parts off at the ends of an item.  In the even slot of an
            // iteration the value addresses move on to the iteration's tile once the update has requested its last
            // fragment; `extra(m)` is further work for the step of MFMA m = 0..31.
            auto slot_fn = [&](auto par_c, auto pv_c, auto sm_c, auto ch_c, int tile, auto extra) {
                constexpr int par = decltype(par_c)::value;
                constexpr bool PV = decltype(pv_c)::value, SM = decltype(sm_c)::value, CH = decltype(ch_c)::value;
                // first part: 16 MFMAs of the O^T update, value fragment i = (kk, dvt) feeds both row blocks
#pragma unroll
                for (int i = 0; i < 2 * NDV; ++i) {
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        LCA_FENCE();
                        // (assembly: keeps O^T in the accumulation registers in every block of the loop)
                        if (PV && F16) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc[rb][i % NDV]) : "v"(vf[i % RING]), "v"(pb[1 - par][rb].v[i / NDV]));
                        if (PV && !F16) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[rb][i % NDV]) : "v"(vf[i % RING]), "v"(pb[1 - par][rb].v[i / NDV]));
                        LCA_FENCE();        // the MFMA first, then this step's other work (left alone, the scheduler puts every second MFMA
                                            // behind its step's work, and the matrix core idles between the pairs)
                        if (rb == 1) {
                            if (PV && i + RING < 2 * NDV) vf[i % RING] = load_v(a, 1 - par, i + RING);
                            if (PV && par == 0 && i == 2 * NDV - RING) {       // the last value fragment of tile `tile`-1 is requested
                                const int d = next_stage(tile - 1);
#pragma unroll
                                for (int t = 0; t < NDV; ++t) a.v[t] += d;
                            }
                            // the chain's first key fragments
                            if (CH && i >= 2 * NDV - RING) kf[i % RING] = load_k(a, 1 - par, i - (2 * NDV - RING));
                        }
                        if (SM) softmax_after(par, 2 * i + rb);
                        extra(2 * i + rb);
                    }
                }
                // second part: 16 MFMAs of the S^T chain, key fragment ks feeds both row blocks
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) {
                        LCA_FENCE();
                        if (CH) chain_mfma(1 - par, rb, ks, kf[ks % RING]);
                        LCA_FENCE();
                        if (rb == 1) {
                            if (CH && ks + RING < NKS) kf[ks % RING] = load_k(a, 1 - par, ks + RING);
                            // the next slot's first value fragments: half `par` of the tile the value addresses now point to
                            if (ks >= NKS - RING) vf[ks % RING] = load_v(a, par, ks - (NKS - RING));
                        }
                        if (SM) softmax_after(par, 16 + 2 * ks + rb);
                        extra(16 + 2 * ks + rb);
                    }
                }
                LCA_FENCE();
            };
            typedef std::integral_constant<int, 0> P0;
            typedef std::integral_constant<int, 1> P1;
            typedef std::true_type Y;
            typedef std::false_type N;

            // ---- tile 0 has landed (tiles 1 and 2 may be on their way); S^T chain of half 0 ----
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * COPIES) : "memory");
            __syncthreads();
#pragma unroll
            for (int f = 0; f < RING; ++f) kf[f] = load_k(a, 0, f);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) chain_mfma(0, rb, ks, kf[ks % RING]);
                if (ks + RING < NKS) kf[ks % RING] = load_k(a, 0, ks + RING);
            }
            // the wait states an MFMA result needs before vector instructions may read it (the chains are assembly: the
            // compiler does not know; inside the loop two MFMAs of the next slot stand between a chain and its readers)
            asm volatile("s_nop 15\n\ts_nop 7" : "+v"(s[0][0]), "+v"(s[0][1]));
            // ---- iterations: slot 2T, barrier, slot 2T+1 ----
            auto iteration = [&](auto first_c, int T) {
                constexpr bool FIRST = decltype(first_c)::value;
                const TileInfo ti = tile_info(T);
                prepare_half(0, 0, ti);
                // The even slot also prepares the copy of tile T+3 (past the item's last tile: zeros), which goes where tile T-1
                // was, in its first steps (they carry no softmax work), and moves the key addresses on to tile T+1 once the
                // chain has requested its last fragment.
                CopyCtl cc;
                CopySel sel;
                unsigned vk = 0, vv = 0;
                slot_fn(P0(), std::integral_constant<bool, !FIRST>(), Y(), Y(), T, [&](int m) {      // no half before the first one
                    switch (m) {
                    case 0: copy_step<0>(cc, sel, cur, T + 3, wave, lds0); break;
                    case 1: copy_step<1>(cc, sel, cur, T + 3, wave, lds0); break;
                    case 2: copy_step<2>(cc, sel, cur, T + 3, wave, lds0); break;
                    case 3:
                        copy_step<3>(cc, sel, cur, T + 3, wave, lds0);
                        vk = (lane >> 4) * cc.stride + chunk_k; vv = (lane >> 4) * cc.stride + chunk_v;
                        LCA_PIN_V(vk); LCA_PIN_V(vv);
                        break;
                    default: break;
                    }
                    if (m >= 24 && (m & 1) == 0) {       // steps of k-steps 4..7, row block 0: two key addresses each
                        const int d = next_stage(T), j = (m - 24);
                        a.k[j] += d; a.k[j + 1] += d;
                        LCA_PIN_V(a.k[j]); LCA_PIN_V(a.k[j + 1]);
                    }
                });
                // tile T+1 has landed (tile T+2 may be on its way) and this wavefront's reads of tile T-1 are in registers ...
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"(COPIES) : "memory");
                __syncthreads();      // ... for every wavefront
                prepare_half(1, 1, ti);
                // the odd slot issues the copy in its first steps; past the last tile its chain runs over stale keys: S^T nobody reads
                slot_fn(P1(), Y(), Y(), Y(), T, [&](int m) {
                    if (m < COPIES) issue_copy_dyn(m, cc, vk, vv);
                });
            };
            int t_first = 0;
            asm volatile("" : "+s"(t_first));    // (opaque: with a known zero the compiler turns the flag arithmetic back into comparisons)
            iteration(Y(), t_first);
            for (int T = 1; T < cur.n_tiles; ++T) iteration(N(), T);
            // ---- O^T update of the last half ----
            slot_fn(P0(), Y(), N(), N(), cur.n_tiles, [](int) {});

            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the trailing copies have landed before the stages are reused
            float l_tot[2];
            bool redo = false;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                l_tot[rb] = st.l_run[rb] + __shfl_xor(st.l_run[rb], 32, 64);
                redo |= !(l_tot[rb] <= L_LIMIT) | (F16 && st.p_max[rb] > P_LIMIT_F16);
            }
            // every wavefront is done with the stages; repeat the item if a row sum ran out of range
            if (!__syncthreads_or(pass == 0 && redo)) break;
            {
                // exact row maxima, one tile at a time (no overlap: this path is rare): tile tl goes into stage tl%2 after the
                // barrier of tile tl-1, which every wavefront reaches after its chains over tile tl-2
                m_exact[0] = NEG_BIG; m_exact[1] = NEG_BIG;
                for (int tl = 0; tl < cur.n_tiles; ++tl) {
                    const CopyCtl cc = make_copy(cur, tl, tl & 1, wave, lds0);
                    issue_copy_all(cc, (lane >> 4) * cc.stride + chunk_k, (lane >> 4) * cc.stride + chunk_v);
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    __syncthreads();
                    Addr ax = adr;
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) ax.k[ks] += (tl & 1) * STAGE_BYTES;
                    const TileInfo ti = tile_info(tl);
#pragma unroll
                    for (int half = 0; half < 2; ++half)
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            floatx16 sv;
#pragma unroll
                            for (int r = 0; r < 16; ++r) sv[r] = 0.f;
#pragma unroll
                            for (int ks = 0; ks < NKS; ++ks) {
                                if (F16) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, load_k(ax, half, ks)), __builtin_bit_cast(f16x8, qf[rb][ks]), sv, 0, 0, 0);
                                else sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_k(ax, half, ks), qf[rb][ks], sv, 0, 0, 0);
                            }
                            mask_half(sv, ti.is_rep != 0, cur.mt_row[rb], cur.raw_lo_row[rb], cur.t_row[rb], ti.e0 + 32 * half, G);
                            m_exact[rb] = fmaxf(m_exact[rb], row_max(sv, c, ti.bias));
                        }
                }
                __syncthreads();
                pass = 2;
                issue_first_copies(cur);
            }
        }

        // request the next item's first tiles (stages 0..2) and queries before writing this item's output
        int nu, nqb;
        kidx += n_slots;
        const bool has_next = item(kidx, nu, nqb);
        const int out_b = cur.b, out_h = cur.h, out_t0 = cur.t_w0;
        const int out_t_row[2] = {cur.t_row[0], cur.t_row[1]};
        const float out_m_ref[2] = {st.m_ref[0], st.m_ref[1]};
        float l_tot[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) l_tot[rb] = st.l_run[rb] + __shfl_xor(st.l_run[rb], 32, 64);
        // this item's output rows go through a buffer descriptor: scalar offsets, rows past the sequence's end dropped
        const int rows_valid = min(max(L - out_t0, 0), BMW);
        const __amdgpu_buffer_rsrc_t o_rs = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(kp.O + (((size_t)out_b * L + out_t0) * H + out_h) * D), (short)0, rows_valid > 0 ? ((rows_valid - 1) * H * D + D) * 2 : 0, RSRC_WORD3);
        if (has_next) {
            cur = make_blk(kp, nu, nqb, wave, n);
            issue_first_copies(cur);
            load_q(kp, cur, lane, qf);
        }

        // ---- epilogue: normalise, transpose through this wavefront's 8 KB of stage 3 (four passes: row block x 64 value
        // columns), store rows of 128 B ----
        constexpr int ORS = 64 * 2 + 16;                     // staging row stride (bytes)
        char *obuf = qbuf;
        const int o_voff = ((lane >> 3) * H * D + (lane & 7) * 8) * 2;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const float inv = 1.f / l_tot[rb];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
#pragma unroll
                for (int d2 = 0; d2 < 2; ++d2)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        union { bf16x4 h; f16x4 hf; uint2 u; } o;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (F16) o.hf[i] = (_Float16)(acc[rb][ch * 2 + d2][r4 * 4 + i] * inv);
                            else o.h[i] = (__bf16)(acc[rb][ch * 2 + d2][r4 * 4 + i] * inv);
                        }
                        *reinterpret_cast<uint2 *>(obuf + n * ORS + (d2 * 32 + 8 * r4 + 4 * G) * 2) = o.u;
                    }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int r8 = 0; r8 < 4; ++r8) {                 // one wave-wide store covers eight rows of 128 B
                    const int r = r8 * 8 + (lane >> 3);
                    const uintx4 v = *reinterpret_cast<const uintx4 *>(obuf + r * ORS + (lane & 7) * 16);
                    __builtin_amdgcn_raw_buffer_store_b128(v, o_rs, o_voff, ((rb * 32 + r8 * 8) * H * D + ch * 64) * 2, 0);
                }
                __builtin_amdgcn_wave_barrier();
            }
            if (kp.lse != nullptr && G == 0 && out_t_row[rb] < L)
                kp.lse[((size_t)out_b * L + out_t_row[rb]) * H + out_h] = (out_m_ref[rb] + log2f(l_tot[rb])) * 0.6931471805599453f;
        }
        if (!has_next) break;
        // the next item's queries have been on their way since before the output was written
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        q_to_fragments(qbuf, lane, qf);
    }
}

}  // namespace

// Query heads that share one work item (and with it every K/V tile read): the largest of 4, 2, 1 that divides the heads
// per KV head; the heads of a KV head then form hps / that many groups (7 heads per KV head: seven groups of one).
static int heads_per_item(int hps) { return hps % NW == 0 ? NW : hps % 2 == 0 ? 2 : 1; }

bool attn_gqa64_supported(const Dims &d)
{
    const int hps = d.H / d.S;
    // segment sizes and row offsets travel as 32-bit byte counts
    // ... and item indices are divided with udiv_small
    const int hw = heads_per_item(hps), rows = BMW * (NW / hw);
    const long n_units = (long)d.B * d.S * (hps / hw), n_items = ((long)d.L + rows - 1) / rows * n_units;
    return (d.dtype == LCA_BF16 || d.dtype == LCA_F16) && d.mode == LCA_MODE_GQA && d.d_pool == D && d.d_sel == D && d.scale > 0.f &&
           (long)(d.L + 4 * BN) * d.S * RB < (1l << 32) && (n_items + 8 * GRID) * n_units < (1l << 32) && (long)d.L * d.g < (1l << 31);
}

hipError_t launch_attn_gqa64(const AttnArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    G64Params kp;
    kp.Q = (const uint16_t *)a.Q; kp.K = (const uint16_t *)a.SEL; kp.V = (const uint16_t *)a.POOL;
    kp.k_rep = (const uint16_t *)a.sel_rep; kp.v_rep = (const uint16_t *)a.pool_rep;
    kp.O = (uint16_t *)a.O; kp.lse = a.lse;
    kp.B = d.B; kp.L = d.L; kp.H = d.H; kp.S = d.S; kp.g = d.g; kp.w = d.w; kp.m = d.m; kp.dense = a.dense;
    const int hps = d.H / d.S;
    kp.hw = heads_per_item(hps);
    kp.hgs = hps / kp.hw;
    const int rows = BMW * (NW / kp.hw);
    kp.n_qb = (d.L + rows - 1) / rows;
    kp.n_units = d.B * d.S * kp.hgs;
    auto magic = [](int dv) { return dv > 1 ? (unsigned)((1ull << 32) / (unsigned)dv + 1) : 0u; };
    kp.g_magic = magic(d.g); kp.units_magic = magic(kp.n_units); kp.hgs_magic = magic(kp.hgs); kp.s_magic = magic(d.S);
    kp.scale_log2 = d.scale * 1.4426950408889634f;
    kp.bias_log2 = d.rep_logit_bias * 1.4426950408889634f;
    // persistent grid: one workgroup per CU (a workgroup takes 128 KB of LDS and most of the registers)
    const long items = (long)kp.n_qb * kp.n_units;
    const long cus = persistent_grid();     // <= GRID
    long grid = items < cus ? items : cus;
    grid = (grid + 7) / 8 * 8;
    if (d.dtype == LCA_F16)
        attn_gqa64_kernel<true><<<(unsigned)grid, 64 * NW, 0, st>>>(kp);
    else
        attn_gqa64_kernel<false><<<(unsigned)grid, 64 * NW, 0, st>>>(kp);
    return hipGetLastError();
}

}  // namespace lca
