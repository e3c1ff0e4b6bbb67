// Latent-space condensation kernels (section 4.2 of the paper; Algorithm 1, first step and group loop).
//
//   summary_query_kernel   qbar = mean of the last n_q queries (and of the heads of a set)
//   condense_reg_kernel    one wavefront per group, the group's rows held in registers; scores by
//                          per-lane partial dots + a reduce-scatter butterfly, online softmax over
//                          sub-blocks of <= 8 rows, pooling in-lane, anchor by (score, index) max.
//                          HBM-bound: every C^KV / K^R byte is read once, as 16-byte coalesced loads.
//   condense_generic_kernel  any sizes, scalar loads; fallback for shapes without an instantiation.
//
// gfx950 only (wave64).
#include "lca_internal.h"

namespace lca {
namespace {

constexpr int WAVE = 64;

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even (inputs are finite)
    return (uint16_t)(u >> 16);
}

template <typename T> struct Elt;
template <> struct Elt<uint16_t> {      // bf16 bit patterns
    static constexpr int EPC = 8;        // elements per 16-byte chunk
    __device__ static float ld(const uint16_t *p) { return bf16_bits_to_float(*p); }
    __device__ static void st(uint16_t *p, float v) { *p = float_to_bf16_bits(v); }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static uint4 pack(const float *f)
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)float_to_bf16_bits(f[2 * i]) | ((uint32_t)float_to_bf16_bits(f[2 * i + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Elt<f16_t> {         // fp16 bit patterns
    static constexpr int EPC = 8;
    __device__ static float ld(const f16_t *p) { return f16_bits_to_float(p->bits); }
    __device__ static void st(f16_t *p, float v) { p->bits = float_to_f16_bits(v); }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = f16_bits_to_float((uint16_t)w[i]);
            f[2 * i + 1] = f16_bits_to_float((uint16_t)(w[i] >> 16));
        }
    }
    __device__ static uint4 pack(const float *f)
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)float_to_f16_bits(f[2 * i]) | ((uint32_t)float_to_f16_bits(f[2 * i + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Elt<float> {
    static constexpr int EPC = 4;
    __device__ static float ld(const float *p) { return *p; }
    __device__ static void st(float *p, float v) { *p = v; }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y); f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
    }
    __device__ static uint4 pack(const float *f)
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};

// ---------------------------------------------------------------------------------------------
// Summary query: qbar[b,s,x] = mean over t in [L-n_q, L), h in set s of Q[b,t,h,x].
// One workgroup of 16 wavefronts per (b, s, 64 chunks of 16 bytes): wavefront v takes the (t, h) pairs
// v, v+16, v+32, ... (row addresses are wave-uniform, kept in scalar registers and stepped without
// divisions), each lane keeps up to 16 independent 16-byte loads in flight -- the 256 pairs of 16 queries x
// 16 heads are one round trip to memory --, and the partial sums are merged in a fixed order through LDS
// (deterministic), one output value per thread.
// ---------------------------------------------------------------------------------------------
constexpr int SQ_WAVES = 16;
constexpr int SQ_DEPTH = 16;
template <typename T>
__global__ __launch_bounds__(SQ_WAVES *WAVE) void summary_query_kernel(const T *__restrict__ Q, float *__restrict__ qbar, int L, int H, int S,
                                                                       int d_qk, int n_q)
{
    constexpr int EPC = Elt<T>::EPC;
    __shared__ float part[SQ_WAVES][WAVE][EPC + 1];
    const int n_chunks = d_qk / EPC;
    const int xblocks = (n_chunks + WAVE - 1) / WAVE;
    const int bs = blockIdx.x / xblocks, xb = blockIdx.x % xblocks;
    const int b = bs / S, s = bs % S, hps = H / S;
    const int lane = threadIdx.x & (WAVE - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int chunk = xb * WAVE + lane;
    const int n = n_q * hps;                       // (t, h) pairs, pair u -> t = L - n_q + u / hps, h = s*hps + u % hps
    float acc[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
    if (chunk < n_chunks) {
        const int step_t = SQ_WAVES / hps, step_h = SQ_WAVES % hps;
        int ut = wave / hps, uh = wave % hps;       // pair u = wave + 16 j  ->  (u / hps, u % hps), stepped with carry
        const T *const base = Q + ((size_t)b * L + (L - n_q)) * H * d_qk + (size_t)s * hps * d_qk + chunk * EPC;
        for (int u0 = wave; u0 < n; u0 += SQ_WAVES * SQ_DEPTH) {
            uint4 v[SQ_DEPTH];
#pragma unroll
            for (int i = 0; i < SQ_DEPTH; ++i) {
                const int u = u0 + i * SQ_WAVES;
                v[i] = u < n ? *reinterpret_cast<const uint4 *>(base + ((size_t)ut * H + uh) * d_qk) : make_uint4(0, 0, 0, 0);
                ut += step_t; uh += step_h;
                if (uh >= hps) { uh -= hps; ++ut; }
            }
#pragma unroll
            for (int i = 0; i < SQ_DEPTH; ++i) {
                float f[EPC];
                Elt<T>::unpack(v[i], f);
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[e] += f[e];
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) part[wave][lane][e] = acc[e];
    __syncthreads();
    // thread x sums the 16 partial values of component x % EPC of chunk x / EPC (wavefront order: the same sum on every run)
    const int ol = threadIdx.x / EPC, oe = threadIdx.x % EPC, ochunk = xb * WAVE + ol;
    if (ol < WAVE && ochunk < n_chunks) {
        float t = 0.f;
#pragma unroll
        for (int wv = 0; wv < SQ_WAVES; ++wv) t += part[wv][ol][oe];
        qbar[(size_t)bs * d_qk + ochunk * EPC + oe] = t / (float)n;
    }
}

// ---------------------------------------------------------------------------------------------
// wave helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sum R per-lane partial values across the wave so that lane l ends with the total of value
// (l >> (6 - log2 R)).  log2(R) halving exchanges, then an all-reduce over the remaining lane bits.
template <int R>
__device__ __forceinline__ float wave_reduce_scatter(float (&v)[R], int lane)
{
    int mask = 32;
#pragma unroll
    for (int n = R; n > 1; n >>= 1, mask >>= 1) {
        const bool hi = (lane & mask) != 0;
#pragma unroll
        for (int i = 0; i < n / 2; ++i) {
            const float lo_half = v[i], hi_half = v[i + n / 2];      // (values first: a choice between two array elements
            const float send = hi ? lo_half : hi_half;               // would become an indexed access to the array)
            const float keep = hi ? hi_half : lo_half;
            v[i] = keep + __shfl_xor(send, mask, WAVE);
        }
    }
    float x = v[0];
    for (; mask >= 1; mask >>= 1) x += __shfl_xor(x, mask, WAVE);
    return x;
}

// ---------------------------------------------------------------------------------------------
// Register-resident condensation: one wave per (sequence, KV source, group).
//   pool part : lane l owns 16-byte chunk l of every row of the sub-block (R <= 8 rows in registers)
//   sel part  : lane l owns row (l >> SH) and every (64/R)-th chunk of it, so its partial dot already
//               sits with the lane that receives that row's score from the reduce-scatter
// ---------------------------------------------------------------------------------------------
template <typename T, int DP, int DS, int G, bool MLA, bool HOLD>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(HOLD ? 2 : 3, 8)))
void condense_reg_kernel(const T *__restrict__ POOL, const T *__restrict__ SEL, const float *__restrict__ qbar,
                         T *__restrict__ pool_rep, T *__restrict__ sel_rep, int32_t *__restrict__ anchor,
                         float *__restrict__ alpha_dbg, int B, int L, int S, int m, float scale)
{
    constexpr int EPC = Elt<T>::EPC;
    constexpr int NCP = DP / EPC, NCS = DS / EPC;
    constexpr int R = G < 8 ? G : 8;            // rows per sub-block (8 keeps three wavefronts per SIMD resident)
    constexpr int NSB = G / R;
    constexpr int LOG2R = R == 8 ? 3 : R == 4 ? 2 : R == 2 ? 1 : 0;
    constexpr int SH = 6 - LOG2R;               // lane l holds the score of sub-block row l >> SH
    constexpr int LPR = 1 << SH;                // lanes per row for the sel part
    constexpr int SPL = (NCS + LPR - 1) / LPR;  // sel chunks per lane
    constexpr int DQK = MLA ? DP + DS : DS;
    static_assert(G % R == 0 && DP % EPC == 0 && DS % EPC == 0 && NCP <= WAVE, "shape");

    const int lane = threadIdx.x & (WAVE - 1);
    const long wave_id = (long)blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x / WAVE);
    const int P = MLA ? 1 : S;                  // KV sources per sequence
    const long n_units = (long)B * P * m;
    if (wave_id >= n_units) return;             // whole wave leaves together
    // the KV sources of a group are neighbours in the unit order: the P wavefronts that read the P interleaved parts of the
    // same g token rows run at the same time, and the rows are fetched from memory as whole contiguous pieces
    const int p = (int)(wave_id % P), j = (int)((wave_id / P) % m), b = (int)(wave_id / ((long)m * P));

    const T *pool_base = POOL + ((size_t)b * L * P + p) * DP;   // row i at + i * P * DP
    const T *sel_base = SEL + ((size_t)b * L * P + p) * DS;
    const bool has_pool = lane < NCP;
    const int pcol = (has_pool ? lane : 0) * EPC;
    const int my_row = lane >> SH, sub = lane & (LPR - 1);

    // the loads of sub-block sb: R whole pool rows (a chunk per lane) and this lane's chunks of its own sel row
    auto load_sub_block = [&](int sb, uint4 (&pdata)[R], uint4 (&sdata)[SPL]) {
        const int row0 = j * G + sb * R;
#pragma unroll
        for (int r = 0; r < R; ++r)
            pdata[r] = has_pool ? *reinterpret_cast<const uint4 *>(pool_base + (size_t)(row0 + r) * P * DP + pcol) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < SPL; ++i) {
            const int c = sub + i * LPR;
            sdata[i] = c < NCS ? *reinterpret_cast<const uint4 *>(sel_base + (size_t)(row0 + my_row) * P * DS + c * EPC) : make_uint4(0, 0, 0, 0);
        }
    };
    // HOLD (several sets over one latent sequence, at most two sub-blocks): the group is loaded once and stays in
    // registers for every set; otherwise a sub-block is loaded when its turn comes.
    constexpr int NHELD = HOLD ? NSB : 1;
    uint4 pheld[NHELD][R], sheld[NHELD][SPL];
    if constexpr (HOLD) {
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) load_sub_block(sb, pheld[sb], sheld[sb]);
    }

    const int s_begin = MLA ? 0 : p, s_end = MLA ? S : p + 1;
    for (int s = s_begin; s < s_end; ++s) {
        const float *qb = qbar + ((size_t)b * S + s) * DQK;
        float m_run = -INFINITY, l_run = 0.f;
        float acc[EPC];
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
        float best_score = -INFINITY;
        int best_row = 0;
        const size_t unit = ((size_t)b * S + s) * m + j;

        auto sub_block = [&](int sb, const uint4 (&pdata)[R], const uint4 (&sdata)[SPL]) {
            // sel part of the score: this lane's chunks of its own row, summed over the row's lanes
            float ssum = 0.f;
#pragma unroll
            for (int i = 0; i < SPL; ++i) {
                const int c = sub + i * LPR;
                if (c < NCS) {
                    float f[EPC];
                    Elt<T>::unpack(sdata[i], f);
                    const float *qs = qb + (MLA ? DP : 0) + c * EPC;
#pragma unroll
                    for (int e = 0; e < EPC; ++e) ssum = fmaf(f[e], qs[e], ssum);
                }
            }
#pragma unroll
            for (int mask = LPR >> 1; mask >= 1; mask >>= 1) ssum += __shfl_xor(ssum, mask, WAVE);
            float dot = ssum;
            if (MLA) {   // pool part of the score: per-lane partial dots of all rows, reduce-scattered
                float qp[EPC];
#pragma unroll
                for (int e = 0; e < EPC; ++e) qp[e] = has_pool ? qb[pcol + e] : 0.f;
                float part[R];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float f[EPC];
                    Elt<T>::unpack(pdata[r], f);
                    float a = 0.f;
#pragma unroll
                    for (int e = 0; e < EPC; ++e) a = fmaf(f[e], qp[e], a);
                    part[r] = a;
                }
                dot += wave_reduce_scatter<R>(part, lane);
            }
            const float score = scale * dot;              // row my_row of this sub-block
            if (alpha_dbg != nullptr && sub == 0) alpha_dbg[unit * G + sb * R + my_row] = score;   // normalised below
            // sub-block maximum and its lowest row
            float bmax = score;
            int brow = my_row;
#pragma unroll
            for (int mask = 32; mask >= LPR; mask >>= 1) {
                const float os = __shfl_xor(bmax, mask, WAVE);
                const int orow = __shfl_xor(brow, mask, WAVE);
                if (os > bmax || (os == bmax && orow < brow)) { bmax = os; brow = orow; }
            }
            if (bmax > best_score) { best_score = bmax; best_row = sb * R + brow; }   // earlier sub-block wins ties
            // online softmax over sub-blocks (Eq. 6) and weighted pooling (Eq. 7)
            const float m_new = fmaxf(m_run, bmax);
            const float corr = __expf(m_run - m_new);      // 0 on the first sub-block
            const float pmine = __expf(score - m_new);
            l_run *= corr;
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[e] *= corr;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float pr = readlane_f(pmine, r << SH);
                l_run += pr;
                float f[EPC];
                Elt<T>::unpack(pdata[r], f);
#pragma unroll
                for (int e = 0; e < EPC; ++e) acc[e] = fmaf(pr, f[e], acc[e]);
            }
            m_run = m_new;
        };
        if constexpr (HOLD) {
#pragma unroll
            for (int sb = 0; sb < NSB; ++sb) sub_block(sb, pheld[sb], sheld[sb]);
        } else {
#pragma unroll 1
            for (int sb = 0; sb < NSB; ++sb) {
                uint4 pdata[R], sdata[SPL];
                load_sub_block(sb, pdata, sdata);            // every load of the sub-block is issued first
                sub_block(sb, pdata, sdata);
            }
        }

        const float inv_l = 1.f / l_run;
        if (has_pool) {
            float o[EPC];
#pragma unroll
            for (int e = 0; e < EPC; ++e) o[e] = acc[e] * inv_l;
            *reinterpret_cast<uint4 *>(pool_rep + unit * DP + pcol) = Elt<T>::pack(o);
        }
        const int a_tok = j * G + best_row;
        if (lane < NCS)
            *reinterpret_cast<uint4 *>(sel_rep + unit * DS + lane * EPC) =
                *reinterpret_cast<const uint4 *>(sel_base + (size_t)a_tok * P * DS + lane * EPC);
        if (lane == 0) anchor[unit] = a_tok;
        if (alpha_dbg != nullptr && sub == 0) {      // each lane turns the scores it wrote into weights
            for (int sb = 0; sb < NSB; ++sb) {
                float *ap = alpha_dbg + unit * G + sb * R + my_row;
                *ap = __expf(*ap - m_run) * inv_l;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Generic condensation: one wave per (b, s, j), run-time sizes, g <= 64; any reduce strategy for either
// component (the ablation grid of section 5.4, Table 5).
// ---------------------------------------------------------------------------------------------
// Lane r holds v_r (r < g); returns, in every lane, the row with the largest v (lowest row on ties).
__device__ __forceinline__ int wave_argmax(float v, int lane, float *vmax_out)
{
    float bmax = v;
    int brow = lane;
    for (int mask = 32; mask >= 1; mask >>= 1) {
        const float os = __shfl_xor(bmax, mask, WAVE);
        const int orow = __shfl_xor(brow, mask, WAVE);
        if (os > bmax || (os == bmax && orow < brow)) { bmax = os; brow = orow; }
    }
    if (vmax_out) *vmax_out = bmax;
    return brow;
}

// One component of the representative: rows base + (j*g + r)*row_stride, r < g, `width` wide, into out.
//   WEIGHTED / MEAN: sum of w_r x_r with lane r holding w_r;  MAXSEL / MAXPOOL: row `pick`, copied bit for bit.
template <typename T>
__device__ __forceinline__ void reduce_component(int strategy, const T *base, size_t row_stride, int j, int g, int width, float w_mine, int pick,
                                                 T *out, int lane)
{
    if (strategy == LCA_REDUCE_MAXSEL || strategy == LCA_REDUCE_MAXPOOL) {
        const T *src = base + (size_t)(j * g + pick) * row_stride;
        for (int x = lane; x < width; x += WAVE) out[x] = src[x];
        return;
    }
    for (int x0 = 0; x0 < width; x0 += WAVE) {      // every lane takes part in the broadcasts
        const int x = x0 + lane;
        float acc = 0.f;
        for (int r = 0; r < g; ++r) {
            const float wr = __shfl(w_mine, r, WAVE);
            if (x < width) acc = fmaf(wr, Elt<T>::ld(base + (size_t)(j * g + r) * row_stride + x), acc);
        }
        if (x < width) Elt<T>::st(out + x, acc);
    }
}

// Lane r gets the squared Euclidean norm of row r of the group (for MAXPOOL).
template <typename T>
__device__ __forceinline__ float row_norms(const T *base, size_t row_stride, int j, int g, int width, int lane)
{
    float mine = -INFINITY;
    for (int r = 0; r < g; ++r) {
        float a = 0.f;
        for (int x = lane; x < width; x += WAVE) {
            const float v = Elt<T>::ld(base + (size_t)(j * g + r) * row_stride + x);
            a = fmaf(v, v, a);
        }
        for (int mask = 32; mask >= 1; mask >>= 1) a += __shfl_xor(a, mask, WAVE);
        if (lane == r) mine = a;
    }
    return mine;
}

template <typename T>
__global__ __launch_bounds__(256) void condense_generic_kernel(const T *__restrict__ POOL, const T *__restrict__ SEL,
                                                               const float *__restrict__ qbar, T *__restrict__ pool_rep,
                                                               T *__restrict__ sel_rep, int32_t *__restrict__ anchor,
                                                               float *__restrict__ alpha_dbg, int B, int L, int S, int m, int g,
                                                               int d_pool, int d_sel, int mla, float scale, int pool_reduce, int sel_reduce)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const long unit = (long)blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x / WAVE);
    if (unit >= (long)B * S * m) return;
    const int j = (int)(unit % m), s = (int)((unit / m) % S), b = (int)(unit / ((long)m * S));
    const int P = mla ? 1 : S, p = mla ? 0 : s, d_qk = mla ? d_pool + d_sel : d_sel;
    const float *qb = qbar + ((size_t)b * S + s) * d_qk;
    const T *pool_base = POOL + ((size_t)b * L * P + p) * d_pool;
    const T *sel_base = SEL + ((size_t)b * L * P + p) * d_sel;
    const size_t pool_stride = (size_t)P * d_pool, sel_stride = (size_t)P * d_sel;

    float my_score = -INFINITY;            // lane r holds the score of row r
    for (int r = 0; r < g; ++r) {
        const T *pr = pool_base + (size_t)(j * g + r) * pool_stride;
        const T *sr = sel_base + (size_t)(j * g + r) * sel_stride;
        float a = 0.f;
        if (mla)
            for (int x = lane; x < d_pool; x += WAVE) a = fmaf(Elt<T>::ld(pr + x), qb[x], a);
        const int qoff = mla ? d_pool : 0;
        for (int x = lane; x < d_sel; x += WAVE) a = fmaf(Elt<T>::ld(sr + x), qb[qoff + x], a);
        for (int mask = 32; mask >= 1; mask >>= 1) a += __shfl_xor(a, mask, WAVE);
        if (lane == r) my_score = scale * a;
    }
    float bmax;
    const int brow = wave_argmax(my_score, lane, &bmax);
    const float pmine = lane < g ? __expf(my_score - bmax) : 0.f;
    float z = pmine;
    for (int mask = 32; mask >= 1; mask >>= 1) z += __shfl_xor(z, mask, WAVE);
    const float alpha = pmine / z;
    const float mean_w = lane < g ? 1.f / (float)g : 0.f;

    int pick_pool = brow, pick_sel = brow;
    if (pool_reduce == LCA_REDUCE_MAXPOOL) pick_pool = wave_argmax(row_norms(pool_base, pool_stride, j, g, d_pool, lane), lane, nullptr);
    if (sel_reduce == LCA_REDUCE_MAXPOOL) pick_sel = wave_argmax(row_norms(sel_base, sel_stride, j, g, d_sel, lane), lane, nullptr);
    reduce_component(pool_reduce, pool_base, pool_stride, j, g, d_pool, pool_reduce == LCA_REDUCE_MEAN ? mean_w : alpha, pick_pool,
                     pool_rep + (size_t)unit * d_pool, lane);
    reduce_component(sel_reduce, sel_base, sel_stride, j, g, d_sel, sel_reduce == LCA_REDUCE_MEAN ? mean_w : alpha, pick_sel,
                     sel_rep + (size_t)unit * d_sel, lane);
    if (lane == 0) anchor[unit] = j * g + brow;
    if (alpha_dbg != nullptr && lane < g) alpha_dbg[(size_t)unit * g + lane] = alpha;
}

template <typename T, int DP, int DS, int G, bool MLA>
hipError_t run_reg(const CondenseArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    const long units = (long)d.B * (MLA ? 1 : d.S) * d.m;
    const int blocks = (int)((units + 3) / 4);
    if constexpr (MLA && G <= 16) {
        if (d.S > 1) {       // every set reads the same group: it is kept in registers across the sets
            condense_reg_kernel<T, DP, DS, G, MLA, true><<<blocks, 256, 0, st>>>(
                (const T *)a.POOL, (const T *)a.SEL, a.qbar, (T *)a.pool_rep, (T *)a.sel_rep, a.anchor, a.alpha_dbg, d.B, d.L, d.S, d.m, d.scale);
            return hipGetLastError();
        }
    }
    condense_reg_kernel<T, DP, DS, G, MLA, false><<<blocks, 256, 0, st>>>(
        (const T *)a.POOL, (const T *)a.SEL, a.qbar, (T *)a.pool_rep, (T *)a.sel_rep, a.anchor, a.alpha_dbg, d.B, d.L, d.S, d.m, d.scale);
    return hipGetLastError();
}

template <typename T>
hipError_t run_generic(const CondenseArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    const long units = (long)d.B * d.S * d.m;
    const int blocks = (int)((units + 3) / 4);
    condense_generic_kernel<T><<<blocks, 256, 0, st>>>((const T *)a.POOL, (const T *)a.SEL, a.qbar, (T *)a.pool_rep, (T *)a.sel_rep,
                                                       a.anchor, a.alpha_dbg, d.B, d.L, d.S, d.m, d.g, d.d_pool, d.d_sel,
                                                       d.mode == LCA_MODE_MLA, d.scale, d.pool_reduce, d.sel_reduce);
    return hipGetLastError();
}

template <typename T, int DP, int DS, bool MLA>
bool try_reg(const CondenseArgs &a, hipStream_t st, hipError_t &err)
{
    switch (a.d.g) {
    case 1: err = run_reg<T, DP, DS, 1, MLA>(a, st); return true;
    case 2: err = run_reg<T, DP, DS, 2, MLA>(a, st); return true;
    case 4: err = run_reg<T, DP, DS, 4, MLA>(a, st); return true;
    case 8: err = run_reg<T, DP, DS, 8, MLA>(a, st); return true;
    case 16: err = run_reg<T, DP, DS, 16, MLA>(a, st); return true;
    case 32: err = run_reg<T, DP, DS, 32, MLA>(a, st); return true;
    default: return false;
    }
}

}  // namespace

// qbar [B,S,d_qk] = mean of the last n_q of the L queries in Q [B,L,H,d_qk] (and of each set's heads)
hipError_t launch_summary_query(const Dims &d, const void *Q, int L, float *qbar, hipStream_t st)
{
    if (d.dtype == LCA_BF16) {
        const int sq_blocks = d.B * d.S * ((d.d_qk / 8 + WAVE - 1) / WAVE);
        summary_query_kernel<uint16_t><<<sq_blocks, SQ_WAVES * WAVE, 0, st>>>((const uint16_t *)Q, qbar, L, d.H, d.S, d.d_qk, d.n_q);
    } else if (d.dtype == LCA_F16) {
        const int sq_blocks = d.B * d.S * ((d.d_qk / 8 + WAVE - 1) / WAVE);
        summary_query_kernel<f16_t><<<sq_blocks, SQ_WAVES * WAVE, 0, st>>>((const f16_t *)Q, qbar, L, d.H, d.S, d.d_qk, d.n_q);
    } else {
        const int sq_blocks = d.B * d.S * ((d.d_qk / 4 + WAVE - 1) / WAVE);
        summary_query_kernel<float><<<sq_blocks, SQ_WAVES * WAVE, 0, st>>>((const float *)Q, qbar, L, d.H, d.S, d.d_qk, d.n_q);
    }
    return hipGetLastError();
}

hipError_t launch_condense(const CondenseArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    // 1. summary query (Algorithm 1, first step)
    hipError_t err = launch_summary_query(d, a.Q, d.L, a.qbar, st);
    if (err != hipSuccess || d.m == 0) return err;
    // MLA widths, several sets, groups of whole 16-row tiles: scores and pooling on the matrix cores.  (Measured at 128K, g = 16,
    // this kernel / the register kernel below, summary query included: 52 / 40 us with one set, 52 / 51 with two, 55 / 72 with
    // four, 60 / 111 with eight, 72 / 190 with sixteen.)
    if (condense_mla_mfma_supported(d) && d.S >= 3) return launch_condense_mla_mfma(a, st);
    // 2. groups
    const bool mla = d.mode == LCA_MODE_MLA;
    // the register kernels implement the method's own strategies (weighted pooling, max selection); the ablation's others run generic
    auto generic = [&]() {
        return d.dtype == LCA_BF16 ? run_generic<uint16_t>(a, st) : d.dtype == LCA_F16 ? run_generic<f16_t>(a, st) : run_generic<float>(a, st);
    };
    if (d.pool_reduce != LCA_REDUCE_WEIGHTED || d.sel_reduce != LCA_REDUCE_MAXSEL) return generic();
    if (d.dtype == LCA_F16 && mla && d.d_pool == 512 && d.d_sel == 64 && try_reg<f16_t, 512, 64, true>(a, st, err)) return err;
    if (d.dtype == LCA_F16 && !mla && d.d_pool == 128 && d.d_sel == 128 && try_reg<f16_t, 128, 128, false>(a, st, err)) return err;
    if (d.dtype == LCA_BF16 && mla && d.d_pool == 512 && d.d_sel == 64 && try_reg<uint16_t, 512, 64, true>(a, st, err)) return err;
    if (d.dtype == LCA_BF16 && !mla && d.d_pool == 128 && d.d_sel == 128 && try_reg<uint16_t, 128, 128, false>(a, st, err)) return err;
    if (d.dtype == LCA_F32 && mla && d.d_pool == 128 && d.d_sel == 32 && try_reg<float, 128, 32, true>(a, st, err)) return err;
    return generic();
}

}  // namespace lca
