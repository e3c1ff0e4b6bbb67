// Online cache update during decoding (section 4.3 of the paper, "Decoding and Online Cache Update"): the g
// oldest raw tokens of the tail ring are condensed into one more representative — importance scores against
// the mean query of the last n_q tokens (Eq. 6), softmax-weighted pooling of the pooled component (Eq. 7),
// the selected component copied from the arg-max token (Eq. 8; lowest index on ties).
//
// The summary query comes from the condensation's own summary_query_kernel (the g recent queries are a
// sequence of length n_q to it).  Then one workgroup of four wavefronts per (sequence, set): the wavefronts
// split the g rows for the scores, the threads split the columns for the pooled row.  g rows of at most 2 KB
// each — the step is bound by launch latency, not by bandwidth, and runs once every g decode steps.  Any
// widths, both element types, both modes.
#include "lca_internal.h"

namespace lca {
namespace {

template <typename T> struct Elt;
template <> struct Elt<uint16_t> {
    __device__ static float ld(const uint16_t *p) { return __uint_as_float((unsigned)*p << 16); }
    __device__ static void st(uint16_t *p, float v)
    {
        unsigned u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }   // NaN stays NaN
        u += 0x7fffu + ((u >> 16) & 1u);                                                        // round to nearest even
        *p = (uint16_t)(u >> 16);
    }
};
template <> struct Elt<f16_t> {
    __device__ static float ld(const f16_t *p) { return f16_bits_to_float(p->bits); }
    __device__ static void st(f16_t *p, float v) { p->bits = float_to_f16_bits(v); }
};
template <> struct Elt<float> {
    __device__ static float ld(const float *p) { return *p; }
    __device__ static void st(float *p, float v) { *p = v; }
};

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

constexpr int UPD_THREADS = 256;

// dynamic LDS: qbar[d_qk] then score[g]
template <typename T>
__global__ __launch_bounds__(UPD_THREADS) void cache_update_kernel(const float *__restrict__ qbar_g, const T *__restrict__ pool_tail,
                                                                   const T *__restrict__ sel_tail, T *__restrict__ pool_rep,
                                                                   T *__restrict__ sel_rep, int32_t *__restrict__ anchor, int S, int P, int d_pool,
                                                                   int d_sel, int d_qk, int g, int m, int mla, float scale, int m_cap, int k_cap,
                                                                   int k_start)
{
    extern __shared__ float lds[];
    float *qbar = lds, *score = lds + d_qk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, s = blockIdx.x, b = blockIdx.y;
    const int p = mla ? 0 : s;
    for (int col = tid; col < d_qk; col += UPD_THREADS) qbar[col] = qbar_g[((size_t)b * S + s) * d_qk + col];
    __syncthreads();

    auto ring_row = [&](int i) { const int r = k_start + i; return r >= k_cap ? r - k_cap : r; };
    const T *ptail = pool_tail + ((size_t)b * P + p) * k_cap * d_pool;
    const T *stail = sel_tail + ((size_t)b * P + p) * k_cap * d_sel;

    // scores of the g oldest tail tokens: key = [pooled ; selected] (MLA, absorbed form) or the selected component (GQA)
    for (int i = wave; i < g; i += UPD_THREADS / 64) {
        const int r = ring_row(i);
        float a = 0.f;
        if (mla)
            for (int col = lane; col < d_pool; col += 64) a += qbar[col] * Elt<T>::ld(ptail + (size_t)r * d_pool + col);
        for (int col = lane; col < d_sel; col += 64) a += qbar[(mla ? d_pool : 0) + col] * Elt<T>::ld(stail + (size_t)r * d_sel + col);
        a = wave_sum(a) * scale;
        if (lane == 0) score[i] = a;
    }
    __syncthreads();

    // group softmax and arg-max (every thread redundantly: g <= 64 values)
    float mx = -INFINITY;
    int best = 0;
    for (int i = 0; i < g; ++i)
        if (score[i] > mx) { mx = score[i]; best = i; }
    float z = 0.f;
    for (int i = 0; i < g; ++i) z += __expf(score[i] - mx);
    const float inv_z = 1.f / z;

    // pooled component: softmax-weighted sum; selected component: the arg-max token's, copied
    T *prep = pool_rep + (((size_t)b * S + s) * m_cap + (m - 1)) * d_pool;
    T *srep = sel_rep + (((size_t)b * S + s) * m_cap + (m - 1)) * d_sel;
    for (int col = tid; col < d_pool; col += UPD_THREADS) {
        float a = 0.f;
        for (int i = 0; i < g; ++i) a += __expf(score[i] - mx) * inv_z * Elt<T>::ld(ptail + (size_t)ring_row(i) * d_pool + col);
        Elt<T>::st(prep + col, a);
    }
    const int rb = ring_row(best);
    for (int col = tid; col < d_sel; col += UPD_THREADS) srep[col] = stail[(size_t)rb * d_sel + col];
    if (anchor != nullptr && tid == 0) anchor[((size_t)b * S + s) * m_cap + (m - 1)] = (m - 1) * g + best;
}

template <typename T>
hipError_t run(const UpdateArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    const size_t lds_bytes = (size_t)(d.d_qk + d.g) * sizeof(float);
    cache_update_kernel<T><<<dim3(d.S, d.B), UPD_THREADS, lds_bytes, st>>>(
        a.qbar, (const T *)a.pool_tail, (const T *)a.sel_tail, (T *)a.pool_rep, (T *)a.sel_rep, a.anchor, d.S, d.P, d.d_pool, d.d_sel, d.d_qk, d.g,
        d.m, d.mode == LCA_MODE_MLA ? 1 : 0, d.scale, a.m_cap, a.k_cap, a.k_start);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_cache_update(const UpdateArgs &a, hipStream_t st)
{
    // the n_q recent queries are, to the summary-query kernel, a sequence of n_q tokens of which it averages the last n_q
    const hipError_t e = launch_summary_query(a.d, a.q_recent, a.d.n_q, a.qbar, st);
    if (e != hipSuccess) return e;
    return a.d.dtype == LCA_BF16 ? run<uint16_t>(a, st) : a.d.dtype == LCA_F16 ? run<f16_t>(a, st) : run<float>(a, st);
}

}  // namespace lca
