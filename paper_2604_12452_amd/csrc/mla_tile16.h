// Pieces shared by the kernels that work on tiles of 16 cache rows at the MLA widths (d_c = 512, d_R = 64, 16-bit elements)
// with one wavefront per tile: the LDS layout of a tile, the matrix-core and LDS-transpose instructions for either element
// type, and the direct-to-LDS copies.  Used by the decode step (decode_mla.hip) and by the matrix-core condensation
// (condense_mla_mfma.hip).
#pragma once
#include "lca_internal.h"

namespace lca {
namespace tile16 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// The kernel is a template over the 16-bit element type E (__bf16 or _Float16); these overloads pick the instructions.
__device__ __forceinline__ floatx4 mfma_16x16x32(bf16x8 a, bf16x8 b, floatx4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ floatx4 mfma_16x16x32(f16x8 a, f16x8 b, floatx4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ floatx4 mfma_16x16x16(bf16x4 a, bf16x4 b, floatx4 c)
{
    typedef short shortx4 __attribute__((ext_vector_type(4)));
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, a), __builtin_bit_cast(shortx4, b), c, 0, 0, 0);
}
__device__ __forceinline__ floatx4 mfma_16x16x16(f16x4 a, f16x4 b, floatx4 c) { return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ bf16x4 lds_read_tr16(__attribute__((address_space(3))) bf16x4 *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(p); }
__device__ __forceinline__ f16x4 lds_read_tr16(__attribute__((address_space(3))) f16x4 *p)
{
    typedef __fp16 fp16x4 __attribute__((__vector_size__(4 * sizeof(__fp16))));     // the builtin's own spelling of four halves
    return __builtin_bit_cast(f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4f16((__attribute__((address_space(3))) fp16x4 *)p));
}
// LDS layout of a tile: 16 latent rows of 1 KB at a 1040-byte stride (16-byte reads of 16 rows and transpose reads of rows 4
// apart are both free of bank conflicts), then the 16 RoPE parts of 128 B with their 16-byte chunks XOR-swizzled by row & 7.
constexpr int DP = 512, DS = 64, DQK = 576;
constexpr int BN = 16;                          // entries per tile
constexpr int RSB = 1040;                       // LDS row stride of the latent part: 1024 + 16
constexpr int SEL_OFF = BN * RSB;               // RoPE part: 16 rows x 128 B, chunks swizzled by row & 7
constexpr int BUF_BYTES = SEL_OFF + BN * DS * 2;   // 18 688; two per wavefront
constexpr int COPIES = BN + BN / 8;             // direct-to-LDS loads per 16-bit tile: 18

__device__ __forceinline__ unsigned lds_address(const char *p) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)p; }

// Direct-to-LDS loads of 64 x 16 bytes (lane l -> LDS [lds_addr + 16 l, +16)); inline assembly so that the compiler
// does not tie later LDS reads to them — the wavefront waits for its copies by hand (s_waitcnt vmcnt(0)).
__device__ __forceinline__ void dma_row(unsigned voff, const void *base, unsigned lds_addr)      // uniform base + per-lane offset
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_addr));
}
__device__ __forceinline__ void dma_lanes(const void *addr, unsigned lds_addr)                    // per-lane addresses
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(addr), "s"(lds_addr));
}

}  // namespace tile16
}  // namespace lca
