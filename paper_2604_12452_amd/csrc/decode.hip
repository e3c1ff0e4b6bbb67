// Decode step over a condensed cache (section 4.3, decoding paragraph): one new query per sequence
// and head attends the m representatives and the k raw tail rows.  HBM-bound: every cache byte is
// read once with 16-byte coalesced loads; the query heads of a set share the rows they read.
//
//   decode_split_kernel   one workgroup per (sequence, set, split of the entries): LPR lanes per row,
//                         64/LPR rows per wavefront step, online softmax per lane group, then one
//                         merge per workgroup; writes (max, sum, unnormalised output) partials.
//   decode_merge_kernel   merges the splits and writes O.
// The MLA and GQA layer widths have matrix-core kernels of their own (decode_mla.hip, decode_gqa_mfma.hip), which
// share the merge kernel; decode_split_kernel serves the other instantiated shapes.
#include "lca_internal.h"

namespace lca {
namespace {

constexpr int WAVE = 64;
constexpr int NWAVE = 4;
constexpr int TARGET_BLOCKS = 2048;   // ~8 workgroups per CU

template <typename T> struct DElt;
template <> struct DElt<uint16_t> {
    static constexpr int EPC = 8;
    __device__ static float ld(const uint16_t *p) { return __uint_as_float(((uint32_t)*p) << 16); }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static void st(uint16_t *p, float v)
    {
        uint32_t u = __float_as_uint(v);
        u += 0x7FFFu + ((u >> 16) & 1u);
        *p = (uint16_t)(u >> 16);
    }
};
template <> struct DElt<f16_t> {
    static constexpr int EPC = 8;
    __device__ static float ld(const f16_t *p) { return f16_bits_to_float(p->bits); }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = f16_bits_to_float((uint16_t)w[i]);
            f[2 * i + 1] = f16_bits_to_float((uint16_t)(w[i] >> 16));
        }
    }
    __device__ static void st(f16_t *p, float v) { p->bits = float_to_f16_bits(v); }
};
template <> struct DElt<float> {
    static constexpr int EPC = 4;
    __device__ static float ld(const float *p) { return *p; }
    __device__ static void unpack(const uint4 &c, float *f)
    {
        f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y); f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
    }
    __device__ static void st(float *p, float v) { *p = v; }
};

constexpr int pow2_at_least(int x) { int p = 1; while (p < x) p <<= 1; return p; }

// partial layout in the workspace: [B][S][splits][HPS][DP + 2] floats = (max, sum, acc[DP])
template <typename T, int DP, int DS, bool MLA, int HPS>
__global__ __launch_bounds__(WAVE *NWAVE) void decode_split_kernel(const T *__restrict__ q, const T *__restrict__ pool_rep,
                                                                   const T *__restrict__ sel_rep, const T *__restrict__ pool_tail,
                                                                   const T *__restrict__ sel_tail, float *__restrict__ part, int S, int P,
                                                                   int m, int k, int splits, float scale, float rep_bias, int m_cap,
                                                                   int k_cap, int k_start)
{
    constexpr int EPC = DElt<T>::EPC;
    constexpr int DQK = MLA ? DP + DS : DS;
    constexpr int NCP = DP / EPC, NCS = DS / EPC;
    constexpr int NROW = NCP + NCS;                       // chunks of a [pool | sel] row
    constexpr int LPR = pow2_at_least(NROW) > WAVE ? WAVE : pow2_at_least(NROW);   // lanes per row
    constexpr int RPW = WAVE / LPR;                       // rows per wavefront step
    constexpr int NSLOT = (NROW + LPR - 1) / LPR;
    constexpr int H = HPS;

    __shared__ __attribute__((aligned(16))) T q_s[H * DQK];
    __shared__ float comb[H * (DP + 2)];

    const int tid = threadIdx.x, wave = tid / WAVE, lane = tid % WAVE, sub = lane % LPR, grp = lane / LPR;
    const int split = blockIdx.x % splits, s = (blockIdx.x / splits) % S, b = blockIdx.x / (splits * S);
    const int p = MLA ? 0 : s;
    const int n = m + k;
    const int per = (n + splits - 1) / splits;
    const int e_lo = split * per, e_hi = min(n, e_lo + per);

    for (int x = tid; x < H * DQK; x += WAVE * NWAVE) q_s[x] = q[((size_t)b * S + s) * H * DQK + x];   // heads of set s are contiguous
    __syncthreads();

    bool is_pool[NSLOT], is_sel[NSLOT];
    int col[NSLOT];
#pragma unroll
    for (int sl = 0; sl < NSLOT; ++sl) {
        const int c = sl * LPR + sub;
        is_pool[sl] = c < NCP;
        is_sel[sl] = c >= NCP && c < NROW;
        col[sl] = is_pool[sl] ? c * EPC : (c - NCP) * EPC;
    }

    float mr[H], lr[H], acc[H][NSLOT][EPC];
#pragma unroll
    for (int h = 0; h < H; ++h) {
        mr[h] = -INFINITY;
        lr[h] = 0.f;
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl)
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[h][sl][e] = 0.f;
    }

    for (int base = e_lo + wave * RPW; base < e_hi; base += NWAVE * RPW) {
        const int e = base + grp;
        const bool valid = e < e_hi;
        const int ec = valid ? e : e_hi - 1;
        const T *prow, *srow;
        if (ec < m) {
            prow = pool_rep + (((size_t)b * S + s) * m_cap + ec) * DP;
            srow = sel_rep + (((size_t)b * S + s) * m_cap + ec) * DS;
        } else {
            int r = k_start + (ec - m);                         // the tail is a ring of k_cap rows
            r = r >= k_cap ? r - k_cap : r;
            prow = pool_tail + (((size_t)b * P + p) * k_cap + r) * DP;
            srow = sel_tail + (((size_t)b * P + p) * k_cap + r) * DS;
        }
        uint4 data[NSLOT];
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl) {
            data[sl] = make_uint4(0, 0, 0, 0);
            if (is_pool[sl]) data[sl] = *reinterpret_cast<const uint4 *>(prow + col[sl]);
            else if (is_sel[sl]) data[sl] = *reinterpret_cast<const uint4 *>(srow + col[sl]);
        }
        float f[NSLOT][EPC];
#pragma unroll
        for (int sl = 0; sl < NSLOT; ++sl) DElt<T>::unpack(data[sl], f[sl]);
        float dot[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            float a = 0.f;
#pragma unroll
            for (int sl = 0; sl < NSLOT; ++sl) {
                const bool used = MLA ? (is_pool[sl] || is_sel[sl]) : is_sel[sl];
                if (used) {
                    const int qoff = is_pool[sl] ? col[sl] : (MLA ? DP + col[sl] : col[sl]);
#pragma unroll
                    for (int x = 0; x < EPC; ++x) a = fmaf(f[sl][x], DElt<T>::ld(&q_s[h * DQK + qoff + x]), a);
                }
            }
#pragma unroll
            for (int mask = LPR / 2; mask >= 1; mask >>= 1) a += __shfl_xor(a, mask, WAVE);
            dot[h] = a;
        }
        const float bias = ec < m ? rep_bias : 0.f;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const float logit = valid ? fmaf(dot[h], scale, bias) : -INFINITY;
            const float m_new = fmaxf(mr[h], logit);
            const float m_eff = m_new == -INFINITY ? 0.f : m_new;
            const float corr = __expf(mr[h] - m_eff);
            const float pe = __expf(logit - m_eff);
            lr[h] = lr[h] * corr + pe;
            mr[h] = m_new;
#pragma unroll
            for (int sl = 0; sl < NSLOT; ++sl)
                if (sl * LPR < NCP) {
#pragma unroll
                    for (int x = 0; x < EPC; ++x) acc[h][sl][x] = fmaf(pe, f[sl][x], acc[h][sl][x] * corr);
                }
        }
    }

    // merge the lane groups of this wavefront (they hold the same columns for different rows)
#pragma unroll
    for (int h = 0; h < H; ++h) {
#pragma unroll
        for (int mask = LPR; mask < WAVE; mask <<= 1) {
            const float om = __shfl_xor(mr[h], mask, WAVE), ol = __shfl_xor(lr[h], mask, WAVE);
            const float m_new = fmaxf(mr[h], om);
            const float m_eff = m_new == -INFINITY ? 0.f : m_new;
            const float ca = __expf(mr[h] - m_eff), cb = __expf(om - m_eff);
            lr[h] = lr[h] * ca + ol * cb;
#pragma unroll
            for (int sl = 0; sl < NSLOT; ++sl)
                if (sl * LPR < NCP) {
#pragma unroll
                    for (int x = 0; x < EPC; ++x) acc[h][sl][x] = acc[h][sl][x] * ca + __shfl_xor(acc[h][sl][x], mask, WAVE) * cb;
                }
            mr[h] = m_new;
        }
    }
    // merge the wavefronts one after another through LDS
    for (int wv = 0; wv < NWAVE; ++wv) {
        if (wave == wv && grp == 0) {
#pragma unroll
            for (int h = 0; h < H; ++h) {
                float *cm = comb + h * (DP + 2);
                float ca = 1.f, cb = 0.f, m_new = mr[h], l_new = lr[h];
                if (wv > 0) {
                    const float om = cm[0], ol = cm[1];
                    m_new = fmaxf(mr[h], om);
                    const float m_eff = m_new == -INFINITY ? 0.f : m_new;
                    ca = __expf(mr[h] - m_eff);
                    cb = __expf(om - m_eff);
                    l_new = lr[h] * ca + ol * cb;
                }
#pragma unroll
                for (int sl = 0; sl < NSLOT; ++sl)
                    if (sl * LPR < NCP && is_pool[sl]) {
#pragma unroll
                        for (int x = 0; x < EPC; ++x) {
                            float *dst = cm + 2 + col[sl] + x;
                            *dst = acc[h][sl][x] * ca + (wv > 0 ? *dst * cb : 0.f);
                        }
                    }
                // every lane of the group computed the same (m_new, l_new); write after all lanes have read cm[0..1]
                __builtin_amdgcn_wave_barrier();
                if (sub == 0) { cm[0] = m_new; cm[1] = l_new; }
            }
        }
        __syncthreads();
    }
    float *dst = part + ((((size_t)b * S + s) * splits + split) * H) * (DP + 2);
    for (int x = tid; x < H * (DP + 2); x += WAVE * NWAVE) dst[x] = comb[x];
}

// One workgroup per (b, set, head-in-set): blockIdx.x = (b*S + s)*HPS + h.  The weights of the splits,
// exp(max_sp - max) / sum, are computed once into LDS; then every thread owns two adjacent columns and sums
// the splits' rows with 8-byte loads, eight of them in flight.  DP is even; rows start 8 bytes into a
// (DP + 2)-float record, so 8 bytes is the alignment there is.
constexpr int MERGE_THREADS = 256;
template <typename T>
__global__ __launch_bounds__(MERGE_THREADS) void decode_merge_kernel(const float *__restrict__ part, T *__restrict__ O, int HPS, int DP, int splits)
{
    extern __shared__ float wgt[];                        // [splits]
    __shared__ float red[MERGE_THREADS / WAVE];
    const size_t bs = blockIdx.x / HPS;
    const int h = blockIdx.x % HPS, tid = threadIdx.x;
    const float *base = part + (bs * splits * HPS + h) * (size_t)(DP + 2);
    const size_t stride = (size_t)HPS * (DP + 2);
    auto block_reduce = [&](float v, bool is_max) {
        for (int o = 32; o > 0; o >>= 1) {
            const float u = __shfl_xor(v, o, WAVE);
            v = is_max ? fmaxf(v, u) : v + u;
        }
        __syncthreads();                                  // red[] free again
        if ((tid & (WAVE - 1)) == 0) red[tid / WAVE] = v;
        __syncthreads();
        float r = red[0];
        for (int i = 1; i < MERGE_THREADS / WAVE; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
        return r;
    };
    float mx = -INFINITY;
    for (int sp = tid; sp < splits; sp += MERGE_THREADS) mx = fmaxf(mx, base[sp * stride]);
    mx = block_reduce(mx, true);
    float l = 0.f;
    for (int sp = tid; sp < splits; sp += MERGE_THREADS) {
        const float e = __expf(base[sp * stride] - mx);
        wgt[sp] = e;
        l += base[sp * stride + 1] * e;
    }
    l = block_reduce(l, false);                           // (its barriers also publish wgt[])
    const float inv = 1.f / l;
    for (int x = 2 * tid; x < DP; x += 2 * MERGE_THREADS) {
        float a0 = 0.f, a1 = 0.f;
        const float *col = base + 2 + x;
        int sp = 0;
        for (; sp + 8 <= splits; sp += 8) {
            float2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float2 *>(col + (sp + u) * stride);
#pragma unroll
            for (int u = 0; u < 8; ++u) { a0 = fmaf(v[u].x, wgt[sp + u], a0); a1 = fmaf(v[u].y, wgt[sp + u], a1); }
        }
        for (; sp < splits; ++sp) {
            const float2 v = *reinterpret_cast<const float2 *>(col + sp * stride);
            a0 = fmaf(v.x, wgt[sp], a0);
            a1 = fmaf(v.y, wgt[sp], a1);
        }
        DElt<T>::st(O + (size_t)blockIdx.x * DP + x, a0 * inv);
        DElt<T>::st(O + (size_t)blockIdx.x * DP + x + 1, a1 * inv);
    }
}

template <typename T, int DP, int DS, bool MLA, int HPS>
hipError_t run(const DecodeArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    decode_split_kernel<T, DP, DS, MLA, HPS><<<d.B * d.S * a.splits, WAVE * NWAVE, 0, st>>>(
        (const T *)a.q, (const T *)a.pool_rep, (const T *)a.sel_rep, (const T *)a.pool_tail, (const T *)a.sel_tail, a.part, d.S, d.P, d.m,
        d.k, a.splits, d.scale, d.rep_logit_bias, a.m_cap, a.k_cap, a.k_start);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_merge_kernel<T><<<d.B * d.H, MERGE_THREADS, a.splits * sizeof(float), st>>>(a.part, (T *)a.O, HPS, DP, a.splits);
    return hipGetLastError();
}

// 0 when no instantiation exists
int shape_id(const Dims &d)
{
    const int hps = d.H / d.S;
    const bool mla = d.mode == LCA_MODE_MLA;
    const bool b16 = d.dtype == LCA_BF16 || d.dtype == LCA_F16;    // the 16-bit types share the shapes; the launcher picks the type
    if (b16 && mla && d.d_pool == 512 && d.d_sel == 64 && (hps == 1 || hps == 16)) return 200 + hps;
    if (d.dtype == LCA_F32 && mla && d.d_pool == 128 && d.d_sel == 32 && (hps == 1 || hps == 4)) return 300 + hps;
    return 0;
}

}  // namespace

bool decode_supported(const Dims &d) { return decode_mla_supported(d) || decode_gqa_mfma_supported(d) || shape_id(d) != 0; }

int decode_splits(const Dims &d)
{
    if (decode_mla_supported(d)) return decode_mla_parts(d);
    if (decode_gqa_mfma_supported(d)) return decode_gqa_mfma_parts(d);
    const int n = d.m + d.k;
    int splits = (TARGET_BLOCKS + d.B * d.S - 1) / (d.B * d.S);
    const int max_splits = (n + 63) / 64;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    return splits;
}

size_t decode_workspace_bytes(const Dims &d)
{
    if (!decode_supported(d)) return 0;
    return (size_t)d.B * d.S * decode_splits(d) * (d.H / d.S) * (d.d_pool + 2) * sizeof(float);
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t st)
{
    if (decode_mla_supported(a.d)) {     // matrix-core kernel at the MLA widths, then the common merge
        const hipError_t e = launch_decode_mla(a, st);
        if (e != hipSuccess) return e;
        const int wgs = a.splits / 4;    // one partial result per workgroup of four wavefronts
        if (wgs == 1) return hipSuccess; // ... unless a workgroup had a (sequence, set) to itself: then it wrote O
        if (a.d.dtype == LCA_F16)
            decode_merge_kernel<f16_t><<<a.d.B * a.d.H, MERGE_THREADS, wgs * sizeof(float), st>>>(a.part, (f16_t *)a.O, a.d.H / a.d.S, a.d.d_pool, wgs);
        else
            decode_merge_kernel<uint16_t><<<a.d.B * a.d.H, MERGE_THREADS, wgs * sizeof(float), st>>>(a.part, (uint16_t *)a.O, a.d.H / a.d.S, a.d.d_pool, wgs);
        return hipGetLastError();
    }
    if (decode_gqa_mfma_supported(a.d)) {     // matrix-core kernel at the GQA widths, then the common merge
        const hipError_t e = launch_decode_gqa_mfma(a, st);
        if (e != hipSuccess) return e;
        const int wgs = a.splits / 4;
        if (wgs == 1) return hipSuccess; // a workgroup had a (sequence, KV head) to itself and wrote O
        if (a.d.dtype == LCA_F16)
            decode_merge_kernel<f16_t><<<a.d.B * a.d.H, MERGE_THREADS, wgs * sizeof(float), st>>>(a.part, (f16_t *)a.O, a.d.H / a.d.S, a.d.d_pool, wgs);
        else
            decode_merge_kernel<uint16_t><<<a.d.B * a.d.H, MERGE_THREADS, wgs * sizeof(float), st>>>(a.part, (uint16_t *)a.O, a.d.H / a.d.S, a.d.d_pool, wgs);
        return hipGetLastError();
    }
    const bool f16 = a.d.dtype == LCA_F16;
    switch (shape_id(a.d)) {
    case 201: return f16 ? run<f16_t, 512, 64, true, 1>(a, st) : run<uint16_t, 512, 64, true, 1>(a, st);
    case 216: return f16 ? run<f16_t, 512, 64, true, 16>(a, st) : run<uint16_t, 512, 64, true, 16>(a, st);
    case 301: return run<float, 128, 32, true, 1>(a, st);
    case 304: return run<float, 128, 32, true, 4>(a, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lca
