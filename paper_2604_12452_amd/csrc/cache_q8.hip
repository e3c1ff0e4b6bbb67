// 8-bit storage of the condensed representatives.  The paper's limitations section leaves formats below 16 bits
// open; the format here is this library's: OCP FP8 E4M3 codes (what gfx950's conversion instructions and matrix
// cores speak natively) with one power-of-two scale per representative row and component (pooled part, selected
// part), chosen so that the row's largest magnitude lands in (224, 448].  A power-of-two scale makes x / scale
// exact, so the only rounding is the conversion's (nearest, ties to even).
//
// quantize_kernel: one wavefront per representative row; lane l holds 8 consecutive elements of every 512-element
// slice, the row maximum is a wavefront reduction, the codes leave as one 8-byte store per lane.
#include "lca_internal.h"

namespace lca {
namespace {

template <typename T> __device__ __forceinline__ void unpack8(const uint4 &c, float *f);
template <> __device__ __forceinline__ void unpack8<uint16_t>(const uint4 &c, float *f)
{
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}
template <> __device__ __forceinline__ void unpack8<f16_t>(const uint4 &c, float *f)
{
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = f16_bits_to_float((uint16_t)w[i]);
        f[2 * i + 1] = f16_bits_to_float((uint16_t)(w[i] >> 16));
    }
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// exponent e of the power-of-two scale 2^e for a row whose largest magnitude is amax (0 for an all-zero row)
__device__ __forceinline__ int scale_exponent(float amax)
{
    if (amax == 0.f) return 0;
    int e;
    const float f = frexpf(amax, &e);              // amax = f * 2^e, f in [0.5, 1); 448 = 0.875 * 2^9
    return f <= 0.875f ? e - 9 : e - 8;
}

// one component (width d <= 1024, a multiple of 8) of one row: codes to dst, the scale returned
template <typename T>
__device__ __forceinline__ float quantize_component(const T *src, uint8_t *dst, int d, int lane)
{
    float f[2][8];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int x = c * 512 + lane * 8;
        if (x < d) {
            unpack8<T>(*reinterpret_cast<const uint4 *>(src + x), f[c]);
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[c][i]));
        }
    }
    amax = wave_max(amax);
    const int e = scale_exponent(amax);
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int x = c * 512 + lane * 8;
        if (x < d) {
#pragma unroll
            for (int i = 0; i < 8; ++i) f[c][i] = ldexpf(f[c][i], -e);     // exact
            uint2 out;
            unsigned w = 0;
            w = __builtin_amdgcn_cvt_pk_fp8_f32(f[c][0], f[c][1], w, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(f[c][2], f[c][3], w, true);
            out.x = w;
            w = 0;
            w = __builtin_amdgcn_cvt_pk_fp8_f32(f[c][4], f[c][5], w, false);
            w = __builtin_amdgcn_cvt_pk_fp8_f32(f[c][6], f[c][7], w, true);
            out.y = w;
            *reinterpret_cast<uint2 *>(dst + x) = out;
        }
    }
    return ldexpf(1.f, e);
}

template <typename T>
__global__ __launch_bounds__(256) void quantize_kernel(const T *__restrict__ pool_rep, const T *__restrict__ sel_rep,
                                                       uint8_t *__restrict__ pool_q8, uint8_t *__restrict__ sel_q8,
                                                       float *__restrict__ scales, int first, int n, int m_cap, int sets, int d_pool,
                                                       int d_sel)
{
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);        // over (set, row in [first, first + n)) pairs
    if (row >= (long)sets * n) return;
    const long r = (row / n) * m_cap + first + row % n;                // row of the allocated buffers
    const float sp = quantize_component<T>(pool_rep + r * d_pool, pool_q8 + r * d_pool, d_pool, lane);
    const float ss = quantize_component<T>(sel_rep + r * d_sel, sel_q8 + r * d_sel, d_sel, lane);
    if (lane == 0) {
        scales[2 * r] = sp;
        scales[2 * r + 1] = ss;
    }
}

}  // namespace

hipError_t launch_quantize_cache(const QuantArgs &a, hipStream_t st)
{
    const Dims &d = a.d;
    const int n = d.m - a.first_row;
    if (n <= 0) return hipSuccess;
    const long rows = (long)d.B * d.S * n;
    const unsigned grid = (unsigned)((rows + 3) / 4);
    if (d.dtype == LCA_F16)
        quantize_kernel<f16_t><<<grid, 256, 0, st>>>((const f16_t *)a.pool_rep, (const f16_t *)a.sel_rep, a.pool_q8, a.sel_q8, a.scales, a.first_row, n,
                                                     a.m_cap, d.B * d.S, d.d_pool, d.d_sel);
    else
        quantize_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t *)a.pool_rep, (const uint16_t *)a.sel_rep, a.pool_q8, a.sel_q8, a.scales, a.first_row,
                                                        n, a.m_cap, d.B * d.S, d.d_pool, d.d_sel);
    return hipGetLastError();
}

}  // namespace lca
