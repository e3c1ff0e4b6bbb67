// 8-bit storage of the condensed representatives.  The paper's limitations section leaves formats below 16 bits
// open; the format here is this library's: OCP FP8 E4M3 codes (what gfx950's conversion instructions and matrix
// cores speak natively) with one power-of-two scale per representative row and component (pooled part, selected
// part), chosen so that the row's largest magnitude lands in (224, 448].  A power-of-two scale makes x / scale
// exact, so the only rounding is the conversion's (nearest, ties to even).
//
// quantize_narrow_kernel (widths 8 << l, l <= 6: every layer width here): a row's 8-element pieces sit in 1 << l lanes,
// a wavefront takes 64 >> l rows at once, the row maximum is a reduction over those lanes, the codes leave as one
// 8-byte store per lane.  quantize_kernel (any other width): one wavefront per row.
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

// Any width: one wavefront per row, both components.
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

// One component whose width is 8 << LOG2_LPR elements (8 .. 512): LPR = 1 << LOG2_LPR lanes hold a row, 8 elements each,
// and a wavefront takes 64 / LPR rows at once (a 128-wide row keeps only 16 lanes busy in the kernel above).
template <typename T, int LOG2_LPR>
__global__ __launch_bounds__(256) void quantize_narrow_kernel(const T *__restrict__ src, uint8_t *__restrict__ dst, float *__restrict__ scales,
                                                              int comp, int first, int n, int m_cap, int sets)
{
    constexpr int LPR = 1 << LOG2_LPR, RPW = 64 / LPR, DW = 8 * LPR;
    const int lane = threadIdx.x & 63, sub = lane & (LPR - 1);
    const long row = ((long)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + (lane >> LOG2_LPR);
    const bool live = row < (long)sets * n;
    const long rc = live ? row : 0;
    const long r = (rc / n) * m_cap + first + rc % n;
    float f[8];
    unpack8<T>(*reinterpret_cast<const uint4 *>(src + r * DW + sub * 8), f);
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
    const int e = scale_exponent(amax);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = ldexpf(f[i], -e);               // exact
    uint2 out;
    unsigned w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], w, true);
    out.x = w;
    w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], w, true);
    out.y = w;
    if (live) {
        *reinterpret_cast<uint2 *>(dst + r * DW + sub * 8) = out;
        if (sub == 0) scales[2 * r + comp] = ldexpf(1.f, e);
    }
}

template <typename T, int LOG2_LPR>
void run_narrow(const T *src, uint8_t *dst, float *scales, int comp, const QuantArgs &a, int n, hipStream_t st)
{
    const long rows = (long)a.d.B * a.d.S * n;
    const long waves = (rows * (1 << LOG2_LPR) + 63) / 64;
    quantize_narrow_kernel<T, LOG2_LPR><<<(unsigned)((waves + 3) / 4), 256, 0, st>>>(src, dst, scales, comp, a.first_row, n, a.m_cap, a.d.B * a.d.S);
}

// log2 of the lanes per row if the width is 8 << that (8 .. 512), else -1
int narrow_log2(int d)
{
    for (int l = 0; l <= 6; ++l)
        if (d == (8 << l)) return l;
    return -1;
}

template <typename T>
void run_component(const void *src, uint8_t *dst, float *scales, int comp, int d, const QuantArgs &a, int n, hipStream_t st)
{
    switch (narrow_log2(d)) {
    case 0: run_narrow<T, 0>((const T *)src, dst, scales, comp, a, n, st); break;
    case 1: run_narrow<T, 1>((const T *)src, dst, scales, comp, a, n, st); break;
    case 2: run_narrow<T, 2>((const T *)src, dst, scales, comp, a, n, st); break;
    case 3: run_narrow<T, 3>((const T *)src, dst, scales, comp, a, n, st); break;
    case 4: run_narrow<T, 4>((const T *)src, dst, scales, comp, a, n, st); break;
    case 5: run_narrow<T, 5>((const T *)src, dst, scales, comp, a, n, st); break;
    default: run_narrow<T, 6>((const T *)src, dst, scales, comp, a, n, st); break;
    }
}

template <typename T>
hipError_t run_quantize(const QuantArgs &a, int n, hipStream_t st)
{
    const Dims &d = a.d;
    if (narrow_log2(d.d_pool) >= 0 && narrow_log2(d.d_sel) >= 0) {
        run_component<T>(a.pool_rep, a.pool_q8, a.scales, 0, d.d_pool, a, n, st);
        run_component<T>(a.sel_rep, a.sel_q8, a.scales, 1, d.d_sel, a, n, st);
    } else {
        const long rows = (long)d.B * d.S * n;
        quantize_kernel<T><<<(unsigned)((rows + 3) / 4), 256, 0, st>>>((const T *)a.pool_rep, (const T *)a.sel_rep, a.pool_q8, a.sel_q8, a.scales,
                                                                      a.first_row, n, a.m_cap, d.B * d.S, d.d_pool, d.d_sel);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quantize_cache(const QuantArgs &a, hipStream_t st)
{
    const int n = a.d.m - a.first_row;
    if (n <= 0) return hipSuccess;
    return a.d.dtype == LCA_F16 ? run_quantize<f16_t>(a, n, st) : run_quantize<uint16_t>(a, n, st);
}

}  // namespace lca
