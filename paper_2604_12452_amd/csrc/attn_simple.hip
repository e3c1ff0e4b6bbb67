// Straightforward attention kernel for any sizes and both element types: one wavefront per
// (sequence, token, head) row, fp32 arithmetic, online softmax over chunks of 64 entries.
// Serves the fp32 configuration and every shape the MFMA kernel has no instantiation for.
//
// Row t attends representatives j < m_t and raw tokens m_t*g <= i <= t (section 4.3, Eq. 10 with the
// per-query partition of appendix A.2), or every token i <= t in dense mode (section 3, Eq. 5).
#include "lca_internal.h"

namespace lca {
namespace {

constexpr int WAVE = 64;
constexpr int MAXD = 1024;   // largest d_qk / d_v handled (validated by the API)

template <typename T> __device__ __forceinline__ float ldf(const T *p);
template <> __device__ __forceinline__ float ldf<uint16_t>(const uint16_t *p) { return __uint_as_float(((uint32_t)*p) << 16); }
template <> __device__ __forceinline__ float ldf<f16_t>(const f16_t *p) { return f16_bits_to_float(p->bits); }
template <> __device__ __forceinline__ float ldf<float>(const float *p) { return *p; }

template <typename T> __device__ __forceinline__ void stf(T *p, float v);
template <> __device__ __forceinline__ void stf<uint16_t>(uint16_t *p, float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}
template <> __device__ __forceinline__ void stf<f16_t>(f16_t *p, float v) { p->bits = float_to_f16_bits(v); }
template <> __device__ __forceinline__ void stf<float>(float *p, float v) { *p = v; }

template <typename T>
__global__ __launch_bounds__(WAVE) void attn_simple_kernel(const T *__restrict__ Q, const T *__restrict__ POOL, const T *__restrict__ SEL,
                                                           const T *__restrict__ pool_rep, const T *__restrict__ sel_rep,
                                                           T *__restrict__ O, float *__restrict__ lse, int L, int H, int S, int P,
                                                           int d_pool, int d_sel, int mla, int g, int w, int m, int dense,
                                                           float scale, float rep_bias)
{
    __shared__ float q_s[MAXD];
    __shared__ float p_s[WAVE];
    const int lane = threadIdx.x;
    const long row = blockIdx.x;                 // ((b * L) + t) * H + h
    const int h = (int)(row % H), t = (int)((row / H) % L), b = (int)(row / ((long)H * L));
    const int s = h / (H / S), p = mla ? 0 : s;
    const int d_qk = mla ? d_pool + d_sel : d_sel;
    const int NV = (d_pool + WAVE - 1) / WAVE;   // output columns per lane (<= 16)

    for (int x = lane; x < d_qk; x += WAVE) q_s[x] = ldf(Q + (size_t)row * d_qk + x);
    __syncthreads();

    const int mt = (dense || t + 1 <= w) ? 0 : (t + 1 - w) / g;     // visible representatives
    const int n_raw = t + 1 - mt * g;
    const int n = mt + n_raw;

    float acc[MAXD / WAVE];
#pragma unroll
    for (int i = 0; i < MAXD / WAVE; ++i) acc[i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    for (int e0 = 0; e0 < n; e0 += WAVE) {
        const int e = e0 + lane;
        float logit = -INFINITY;
        const T *vrow = nullptr;
        if (e < n) {
            const T *prow, *srow;
            float bias = 0.f;
            if (e < mt) {
                const size_t r = ((size_t)b * S + s) * m + e;
                prow = pool_rep + r * d_pool;
                srow = sel_rep + r * d_sel;
                bias = rep_bias;
            } else {
                const size_t i = (size_t)(mt * g + (e - mt));
                prow = POOL + (((size_t)b * L + i) * P + p) * d_pool;
                srow = SEL + (((size_t)b * L + i) * P + p) * d_sel;
            }
            float a = 0.f;
            if (mla)
                for (int x = 0; x < d_pool; ++x) a = fmaf(q_s[x], ldf(prow + x), a);
            const int qoff = mla ? d_pool : 0;
            for (int x = 0; x < d_sel; ++x) a = fmaf(q_s[qoff + x], ldf(srow + x), a);
            logit = scale * a + bias;
            vrow = prow;
        }
        float cmax = logit;
        for (int mask = 32; mask >= 1; mask >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, mask, WAVE));
        const float m_new = fmaxf(m_run, cmax);         // finite: every chunk holds at least one entry
        const float corr = __expf(m_run - m_new);
        const float pe = e < n ? __expf(logit - m_new) : 0.f;
        float psum = pe;
        for (int mask = 32; mask >= 1; mask >>= 1) psum += __shfl_xor(psum, mask, WAVE);
        l_run = l_run * corr + psum;
        m_run = m_new;
        __syncthreads();
        p_s[lane] = pe;
        __syncthreads();
        const int cnt = min(WAVE, n - e0);
#pragma unroll
        for (int i = 0; i < MAXD / WAVE; ++i) acc[i] *= corr;
        for (int c = 0; c < cnt; ++c) {
            const unsigned long long vaddr = __shfl((unsigned long long)vrow, c, WAVE);
            const T *vr = reinterpret_cast<const T *>(vaddr);
            const float pc = p_s[c];
#pragma unroll
            for (int i = 0; i < MAXD / WAVE; ++i) {
                const int x = i * WAVE + lane;
                if (i < NV && x < d_pool) acc[i] = fmaf(pc, ldf(vr + x), acc[i]);
            }
        }
    }
    const float inv = 1.f / l_run;
#pragma unroll
    for (int i = 0; i < MAXD / WAVE; ++i) {
        const int x = i * WAVE + lane;
        if (i < NV && x < d_pool) stf(O + (size_t)row * d_pool + x, acc[i] * inv);
    }
    if (lse != nullptr && lane == 0) lse[row] = m_run + __logf(l_run);
}

}  // namespace

hipError_t launch_attn_simple(const AttnArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    const long rows = (long)d.B * d.L * d.H;
    const int mla = d.mode == LCA_MODE_MLA;
    if (d.dtype == LCA_BF16)
        attn_simple_kernel<uint16_t><<<(unsigned)rows, WAVE, 0, st>>>(
            (const uint16_t *)a.Q, (const uint16_t *)a.POOL, (const uint16_t *)a.SEL, (const uint16_t *)a.pool_rep,
            (const uint16_t *)a.sel_rep, (uint16_t *)a.O, a.lse, d.L, d.H, d.S, d.P, d.d_pool, d.d_sel, mla, d.g, d.w, d.m, a.dense,
            d.scale, d.rep_logit_bias);
    else if (d.dtype == LCA_F16)
        attn_simple_kernel<f16_t><<<(unsigned)rows, WAVE, 0, st>>>(
            (const f16_t *)a.Q, (const f16_t *)a.POOL, (const f16_t *)a.SEL, (const f16_t *)a.pool_rep, (const f16_t *)a.sel_rep,
            (f16_t *)a.O, a.lse, d.L, d.H, d.S, d.P, d.d_pool, d.d_sel, mla, d.g, d.w, d.m, a.dense, d.scale, d.rep_logit_bias);
    else
        attn_simple_kernel<float><<<(unsigned)rows, WAVE, 0, st>>>(
            (const float *)a.Q, (const float *)a.POOL, (const float *)a.SEL, (const float *)a.pool_rep, (const float *)a.sel_rep,
            (float *)a.O, a.lse, d.L, d.H, d.S, d.P, d.d_pool, d.d_sel, mla, d.g, d.w, d.m, a.dense, d.scale, d.rep_logit_bias);
    return hipGetLastError();
}

}  // namespace lca
