// Per-token deviations between the original keys / values and the representative that stands for them: the
// delta_k, delta_v of the error bound (section 4.4, Theorem 1 of the paper), measured as in its appendix on
// empirical per-token deviations (Tables 9-10).  HBM-bound: every condensed token's row is read once.
//
//   deviation_group_kernel   one wavefront per (sequence, set, group): lanes stride over the 16-byte pieces of each of the
//                            g rows, wave reductions give || row - rep ||^2 and || row ||^2 for both components;
//                            writes the group's (sum dk, sum dk/||k||, max dk, sum dv, sum dv/||v||, max dv).
//   deviation_reduce_kernel  one workgroup per (sequence, set): adds the groups in a fixed order (deterministic).
#include "lca_internal.h"

namespace lca {
namespace {

constexpr int WAVE = 64;

// 16-byte pieces of a row: EPC elements of type T, widened to float
template <typename T> struct VElt;
template <> struct VElt<uint16_t> {
    static constexpr int EPC = 8;
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
};
template <> struct VElt<f16_t> {
    static constexpr int EPC = 8;
    __device__ static void unpack(const uint4 &c, float *f)
    {
        const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = f16_bits_to_float((uint16_t)w[i]); f[2 * i + 1] = f16_bits_to_float((uint16_t)(w[i] >> 16)); }
    }
};
template <> struct VElt<float> {
    static constexpr int EPC = 4;
    __device__ static void unpack(const uint4 &c, float *f)
    {
        f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y); f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
    }
};

// sum over this lane's 16-byte pieces of (row - rep)^2 and row^2 (widths are multiples of EPC, rows 16-byte aligned: checked at the boundary)
template <typename T>
__device__ __forceinline__ void diff_norms(const T *row, const T *rep, int width, int lane, float &d2, float &n2)
{
    constexpr int EPC = VElt<T>::EPC;
    for (int c = lane; c < width / EPC; c += WAVE) {
        float v[EPC], r[EPC];
        VElt<T>::unpack(*reinterpret_cast<const uint4 *>(row + c * EPC), v);
        VElt<T>::unpack(*reinterpret_cast<const uint4 *>(rep + c * EPC), r);
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            const float x = v[e] - r[e];
            d2 = fmaf(x, x, d2);
            n2 = fmaf(v[e], v[e], n2);
        }
    }
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, WAVE);
    return x;
}

template <typename T>
__global__ __launch_bounds__(256) void deviation_group_kernel(const T *__restrict__ POOL, const T *__restrict__ SEL, const T *__restrict__ pool_rep,
                                                              const T *__restrict__ sel_rep, float *__restrict__ partial, int B, int L, int S, int m,
                                                              int g, int d_pool, int d_sel, int mla)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const long unit = (long)blockIdx.x * (blockDim.x / WAVE) + (threadIdx.x / WAVE);
    if (unit >= (long)B * S * m) return;
    const int j = (int)(unit % m), s = (int)((unit / m) % S), b = (int)(unit / ((long)m * S));
    const int P = mla ? 1 : S, p = mla ? 0 : s;
    const T *pool_base = POOL + ((size_t)b * L * P + p) * d_pool, *sel_base = SEL + ((size_t)b * L * P + p) * d_sel;
    const T *prep = pool_rep + (size_t)unit * d_pool, *srep = sel_rep + (size_t)unit * d_sel;
    float sum_dk = 0.f, sum_rk = 0.f, max_dk = 0.f, sum_dv = 0.f, sum_rv = 0.f, max_dv = 0.f;
    for (int r = 0; r < g; ++r) {
        const T *pr = pool_base + (size_t)(j * g + r) * P * d_pool, *sr = sel_base + (size_t)(j * g + r) * P * d_sel;
        float dp2 = 0.f, np2 = 0.f, ds2 = 0.f, ns2 = 0.f;
        diff_norms(pr, prep, d_pool, lane, dp2, np2);
        diff_norms(sr, srep, d_sel, lane, ds2, ns2);
        dp2 = wave_sum(dp2); np2 = wave_sum(np2); ds2 = wave_sum(ds2); ns2 = wave_sum(ns2);
        const float dk = sqrtf(mla ? dp2 + ds2 : ds2), nk = sqrtf(mla ? np2 + ns2 : ns2), dv = sqrtf(dp2), nv = sqrtf(np2);
        sum_dk += dk; sum_rk += nk > 0.f ? dk / nk : 0.f; max_dk = fmaxf(max_dk, dk);
        sum_dv += dv; sum_rv += nv > 0.f ? dv / nv : 0.f; max_dv = fmaxf(max_dv, dv);
    }
    if (lane == 0) {
        float *o = partial + (size_t)unit * 6;
        o[0] = sum_dk; o[1] = sum_rk; o[2] = max_dk; o[3] = sum_dv; o[4] = sum_rv; o[5] = max_dv;
    }
}

// one workgroup of 256 threads per (sequence, set); groups added in index order within a thread, threads in a fixed tree
__global__ __launch_bounds__(256) void deviation_reduce_kernel(const float *__restrict__ partial, float *__restrict__ stats, int m, int g)
{
    __shared__ float red[256][6];
    const int tid = threadIdx.x;
    const float *base = partial + (size_t)blockIdx.x * m * 6;
    float a[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = tid; j < m; j += 256)
        for (int c = 0; c < 6; ++c) a[c] = (c == 2 || c == 5) ? fmaxf(a[c], base[(size_t)j * 6 + c]) : a[c] + base[(size_t)j * 6 + c];
    for (int c = 0; c < 6; ++c) red[tid][c] = a[c];
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o)
            for (int c = 0; c < 6; ++c) red[tid][c] = (c == 2 || c == 5) ? fmaxf(red[tid][c], red[tid + o][c]) : red[tid][c] + red[tid + o][c];
        __syncthreads();
    }
    if (tid < 6) {
        const float n = m > 0 ? (float)m * (float)g : 1.f;
        stats[(size_t)blockIdx.x * 6 + tid] = (tid == 2 || tid == 5) ? red[0][tid] : red[0][tid] / n;
    }
}

template <typename T>
hipError_t run(const DeviationArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    if (d.m > 0) {
        const long units = (long)d.B * d.S * d.m;
        deviation_group_kernel<T><<<(unsigned)((units + 3) / 4), 256, 0, st>>>((const T *)a.POOL, (const T *)a.SEL, (const T *)a.pool_rep,
                                                                              (const T *)a.sel_rep, a.partial, d.B, d.L, d.S, d.m, d.g, d.d_pool,
                                                                              d.d_sel, d.mode == LCA_MODE_MLA ? 1 : 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    deviation_reduce_kernel<<<d.B * d.S, 256, 0, st>>>(a.partial, a.stats, d.m, d.g);
    return hipGetLastError();
}

}  // namespace

size_t deviation_workspace_bytes(const Dims &d) { return (size_t)d.B * d.S * d.m * 6 * sizeof(float); }

hipError_t launch_deviation_stats(const DeviationArgs &a, hipStream_t st)
{
    return a.d.dtype == LCA_BF16 ? run<uint16_t>(a, st) : a.d.dtype == LCA_F16 ? run<f16_t>(a, st) : run<float>(a, st);
}

}  // namespace lca
