// Measurement aids, not steps of the method: what this chip sustains at the two operations the roofline fractions are read
// against -- streaming a buffer out of HBM once, and back-to-back bf16 matrix-core instructions.  The published peaks (8 TB/s,
// 2.5 PFLOP/s at 2.4 GHz) stay the denominators of every reported fraction; these two say how much of them any kernel can get.
//
//   hbm_read_kernel    persistent grid, 512 threads per workgroup, four 16-byte loads per lane in flight, grid-stride: the launch
//                      shape that read fastest of those tried (256 x 512 x 4 loads: 5.6 TB/s on 151 MB; 8 loads, more or smaller
//                      workgroups: 4.5-5.3).  Every 32-bit word read is added into a per-workgroup sum (mod 2^32), so the reads
//                      cannot be dropped and the result can be checked.
//   mfma_bf16_kernel   one wavefront per SIMD, four independent v_mfma_f32_32x32x16_bf16 chains per wavefront (an instruction
//                      occupies the matrix core for 8 passes of 4 cycles: four chains hide its latency), every chain with operands
//                      of its own.  Pattern 0: small integers -- row i of A is the constant u_i, column j of B the constant v_j, an
//                      output element is 16 iters u_i v_j exactly.  Pattern 1: hashed values with all mantissa bits in use and
//                      mixed signs, like a real kernel's operands: how fast the matrix cores run depends on the clock the chip
//                      settles at, and that on how many operand bits toggle.
#include "lca_internal.h"

namespace lca {
namespace {

constexpr int WAVE = 64;
constexpr int READ_THREADS = 512, READ_UNROLL = 4;

__global__ __launch_bounds__(READ_THREADS) void hbm_read_kernel(const uint4 *__restrict__ p, size_t n16, uint32_t *__restrict__ wg_sums)
{
    __shared__ uint32_t red[READ_THREADS / WAVE];
    const size_t stride = (size_t)gridDim.x * READ_THREADS;
    size_t i = (size_t)blockIdx.x * READ_THREADS + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (READ_UNROLL - 1) * stride < n16; i += READ_UNROLL * stride) {
        uint4 v[READ_UNROLL];
#pragma unroll
        for (int u = 0; u < READ_UNROLL; ++u) v[u] = p[i + u * stride];
#pragma unroll
        for (int u = 0; u < READ_UNROLL; ++u) acc += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    for (; i < n16; i += stride) {
        const uint4 v = p[i];
        acc += v.x + v.y + v.z + v.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, WAVE);
    if ((threadIdx.x & (WAVE - 1)) == 0) red[threadIdx.x / WAVE] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < READ_THREADS / WAVE; ++w) t += red[w];
        wg_sums[blockIdx.x] = t;
    }
}

__global__ void zero_words_kernel(uint32_t *p, int from, int to)
{
    const int i = from + blockIdx.x * blockDim.x + threadIdx.x;
    if (i < to) p[i] = 0;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int CHAINS = 4;

// operand values: integers in [-2, 4] from the lane's row / column index (lane & 31) and the chain; both sums over the 32
// indices are positive for every chain, and 16 iters u v stays below 2^24 for iters <= 65536
__device__ inline int probe_u(int idx, int chain) { return (idx * 5 + chain * 3) % 7 - 2; }
__device__ inline int probe_v(int idx, int chain) { return (idx * 3 + chain * 5 + 1) % 7 - 2; }

// pattern 1: element (idx, k) of operand `which` (0 = A, row idx; 1 = B, column idx) of a chain: sign, one of two exponents and
// 7 mantissa bits from a hash of its coordinates: +-[0.5, 2)
__device__ inline uint32_t probe_hash(uint32_t x)
{
    x *= 2654435761u; x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    return x;
}
__device__ inline uint16_t probe_hashed_bf16(int which, int chain, int idx, int k)
{
    const uint32_t h = probe_hash((uint32_t)(((which * CHAINS + chain) * 32 + idx) * 16 + k) + 1u);
    return (uint16_t)(((h >> 16) & 0x8000u) | ((126u + ((h >> 8) & 1u)) << 7) | (h & 0x7Fu));
}

__global__ __launch_bounds__(256, 1) void mfma_bf16_kernel(int iters, int pattern, float *__restrict__ out)
{
    const int lane = threadIdx.x & (WAVE - 1), idx = lane & 31, k0 = (lane >> 5) * 8;   // A: row idx, B: column idx; k = k0 .. k0 + 7
    bf16x8 a[CHAINS], b[CHAINS];
    f32x16 acc[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) {
        const __bf16 u = (__bf16)(float)probe_u(idx, c), v = (__bf16)(float)probe_v(idx, c);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[c][e] = pattern == 0 ? u : __builtin_bit_cast(__bf16, probe_hashed_bf16(0, c, idx, k0 + e));
            b[c][e] = pattern == 0 ? v : __builtin_bit_cast(__bf16, probe_hashed_bf16(1, c, idx, k0 + e));
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
    }
    // out[thread][chain] = the sum of this lane's 16 output elements of the chain (pattern 0: integers, exact while below 2^24)
#pragma unroll
    for (int c = 0; c < CHAINS; ++c) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[c][e];
        out[((size_t)blockIdx.x * 256 + threadIdx.x) * CHAINS + c] = s;
    }
}

}  // namespace

hipError_t launch_probe_hbm_read(const void *buf, size_t bytes, uint32_t *wg_sums, hipStream_t st)
{
    const int grid = persistent_grid();
    hbm_read_kernel<<<grid, READ_THREADS, 0, st>>>(static_cast<const uint4 *>(buf), bytes / 16, wg_sums);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (grid < LCA_PROBE_WORDS) {
        zero_words_kernel<<<1, LCA_PROBE_WORDS, 0, st>>>(wg_sums, grid, LCA_PROBE_WORDS);
        e = hipGetLastError();
    }
    return e;
}

hipError_t launch_probe_mfma_bf16(int iters, int pattern, float *out, int *wavefronts, hipStream_t st)
{
    const int grid = persistent_grid();
    mfma_bf16_kernel<<<grid, 256, 0, st>>>(iters, pattern, out);
    *wavefronts = grid * (256 / WAVE);
    return hipGetLastError();
}

}  // namespace lca
