// Internal declarations shared by the liblca translation units (host side of the launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lca.h"

namespace lca {

// Element tag of IEEE binary16 storage: the kernels are templates over the element type, bf16 travels as bare
// uint16_t bit patterns, so fp16 gets a distinct 2-byte type of its own.
struct f16_t { uint16_t bits; };
__device__ __forceinline__ float f16_bits_to_float(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t float_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }   // round to nearest even

// Derived sizes of a validated descriptor.
struct Dims {
    int B, L, H, S, P;        // P = KV heads physically present in POOL/SEL (1 for MLA, S for GQA)
    int d_pool, d_sel, d_qk, d_v;
    int g, w, n_q, m, k;      // m groups, k raw tail tokens
    int mode, dtype, elt;     // elt = bytes per element
    float scale, rep_logit_bias;
    int pool_reduce, sel_reduce;   // resolved lca_reduce (never DEFAULT)
};

// Where one attention launch finds its keys/values.
struct AttnArgs {
    Dims d;
    const void *Q, *POOL, *SEL, *pool_rep, *sel_rep;
    void *O;
    float *lse;
    int dense;                // 1: every row sees all tokens i <= t, representatives unused
    const void *W_up = nullptr;   // MLA kernel only: value up-projection [H, 128, d_pool]; O is then [B, L, H, 128]
    void *up_scratch = nullptr;   // ... and H * 128 * d_pool elements of workspace for the matrices in fragment order
};

struct CondenseArgs {
    Dims d;
    const void *Q, *POOL, *SEL;
    void *pool_rep, *sel_rep;
    int32_t *anchor;
    float *alpha_dbg;
    float *qbar;              // workspace, [B, S, d_qk] float
};

struct DecodeArgs {
    Dims d;
    const void *q, *pool_rep, *sel_rep, *pool_tail, *sel_tail;
    const uint8_t *pool_q8 = nullptr, *sel_q8 = nullptr;   // 8-bit representatives instead of pool_rep / sel_rep (MLA widths only)
    const float *scales = nullptr;
    void *O;
    float *part;              // workspace: split partials
    int splits;
    int m_cap, k_cap, k_start;   // rows allocated per (sequence, set) / (sequence, KV head); ring row of the oldest tail token
};

// Online cache update: the g oldest ring rows become representative row m-1.
struct UpdateArgs {
    Dims d;                   // d.m = representatives AFTER the update
    const void *q_recent, *pool_tail, *sel_tail;
    void *pool_rep, *sel_rep;
    int32_t *anchor;
    float *qbar;              // workspace, [B, S, d_qk] float
    int m_cap, k_cap, k_start;
};

// Workgroups of a persistent one-per-CU kernel on the current device (its CU count, a multiple of 8 in [8, 256]).
int persistent_grid();

// Launchers return hipSuccess or the launch error. They assume validated arguments.
hipError_t launch_condense(const CondenseArgs &a, hipStream_t st);
hipError_t launch_summary_query(const Dims &d, const void *Q, int L, float *qbar, hipStream_t st);
// measurement aids (probes.hip)
hipError_t launch_probe_hbm_read(const void *buf, size_t bytes, uint32_t *wg_sums, hipStream_t st);
hipError_t launch_probe_mfma_bf16(int iters, int pattern, float *out, int *wavefronts, hipStream_t st);

bool condense_mla_mfma_supported(const Dims &d);
hipError_t launch_condense_mla_mfma(const CondenseArgs &a, hipStream_t st);
hipError_t launch_attn_simple(const AttnArgs &a, hipStream_t st);
bool attn_mla_supported(const Dims &d);
size_t attn_mla_up_workspace_bytes(const Dims &d);
hipError_t launch_attn_mla(const AttnArgs &a, hipStream_t st);
bool attn_gqa64_supported(const Dims &d);
hipError_t launch_attn_gqa64(const AttnArgs &a, hipStream_t st);
bool decode_supported(const Dims &d);
int decode_splits(const Dims &d);
size_t decode_workspace_bytes(const Dims &d);
hipError_t launch_decode(const DecodeArgs &a, hipStream_t st);
bool decode_mla_supported(const Dims &d);
int decode_mla_parts(const Dims &d);
hipError_t launch_decode_mla(const DecodeArgs &a, hipStream_t st);
bool decode_gqa_mfma_supported(const Dims &d);
int decode_gqa_mfma_parts(const Dims &d);
hipError_t launch_decode_gqa_mfma(const DecodeArgs &a, hipStream_t st);
hipError_t launch_cache_update(const UpdateArgs &a, hipStream_t st);

// 8-bit copy of the representatives in use: codes [.., m_cap, d] and scales [.., m_cap, 2] (pooled, selected).
struct QuantArgs {
    Dims d;
    const void *pool_rep, *sel_rep;
    uint8_t *pool_q8, *sel_q8;
    float *scales;
    int m_cap, first_row;     // rows [first_row, d.m) of every (sequence, set)
};
hipError_t launch_quantize_cache(const QuantArgs &a, hipStream_t st);

// Deviation statistics: per-group partial sums [B,S,m,6] in the workspace, then one reduction per (sequence, set).
struct DeviationArgs {
    Dims d;
    const void *POOL, *SEL, *pool_rep, *sel_rep;
    float *stats, *partial;
};
size_t deviation_workspace_bytes(const Dims &d);
hipError_t launch_deviation_stats(const DeviationArgs &a, hipStream_t st);

}  // namespace lca
