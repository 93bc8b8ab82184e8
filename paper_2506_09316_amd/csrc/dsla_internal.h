// Internal declarations shared by the translation units of libdsla (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "dsla.h"

namespace dsla {

// ---- storage element types -------------------------------------------------------------
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.bits) << 16); }

// fp32 -> bf16, round to nearest even (the hardware conversion of gfx950 does the same).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    __bf16 h = static_cast<__bf16>(f);
    return __builtin_bit_cast(uint16_t, h);
}

template <class T>
__device__ __forceinline__ T from_f32(float f);
template <>
__device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return bf16_t{f32_to_bf16_bits(f)}; }

// ---- profiling hooks (api.hip) -----------------------------------------------------------
// Kernel timing (dsla_profile_enable): a scope reserves a pair of events and the launches inside it carry them in
// the dispatch itself (hipExtLaunchKernelGGL: the start and the end of the kernel are stamped by the dispatch, no
// event packets of their own enter the stream, so timing a launch does not delay the one behind it).  Null events:
// an ordinary launch.
void profile_reserve(int kernel_id, hipEvent_t *start, hipEvent_t *stop);

struct ProfileScope {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipEvent_t e1_first = nullptr;   // the stop event of the first of two launches (set when the second is not issued)
    ProfileScope(int kernel_id, hipStream_t) { profile_reserve(kernel_id, &e0, &e1); }
};
// the only launch of a scope / the first and the last of a scope with two launches
#define DSLA_LAUNCH(ps, kernel, grid, block, shmem, stream, ...)                                                     \
    do {                                                                                                             \
        if ((ps).e0) hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, (ps).e0, (ps).e1, 0, __VA_ARGS__);    \
        else hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                    \
    } while (0)
#define DSLA_LAUNCH_FIRST(ps, kernel, grid, block, shmem, stream, ...)                                               \
    do {                                                                                                             \
        if ((ps).e0) hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, (ps).e0, (ps).e1_first, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                    \
    } while (0)
#define DSLA_LAUNCH_LAST(ps, kernel, grid, block, shmem, stream, ...)                                                \
    do {                                                                                                             \
        if ((ps).e1) hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, nullptr, (ps).e1, 0, __VA_ARGS__);    \
        else hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                    \
    } while (0)

// ---- launchers (one per kernel family; each returns the launch error) ------------------------
hipError_t launch_state_init(float *S1, float *S2, size_t elems_per_state, hipStream_t stream);

// row_index: which row of the token tensors belongs to sequence b (nullptr: row b); state_slot as for the prefill.
hipError_t launch_decode(const dsla_desc &d, const void *q, const void *k, const void *v, const void *g1,
                         const void *g2, const int32_t *row_index, const int32_t *state_slot, float *S1, float *S2,
                         void *o, hipStream_t stream);
bool decode_supported(const dsla_desc &d);

// The per-state pointers and layer-wide blend coefficients of a call with N states, passed to kernels by value.
struct MultiStatePtrs {
    const void *ga[DSLA_MAX_STATES];   // log alpha (or pre-activations) of state n: [..][H][d_k]
    const void *gb[DSLA_MAX_STATES];   // log beta of state n: [..][H][d_v], or null (beta = 1)
    float *S[DSLA_MAX_STATES];         // [slots][H][d_k][d_v]
    float w[DSLA_MAX_STATES];          // blend coefficient of state n
};
hipError_t launch_decode_multi(const dsla_desc &d, const MultiStatePtrs &mp, int N, int Hkv, const float *w_per_head,
                               const void *q, const void *k, const void *v, const int32_t *row_index,
                               const int32_t *state_slot, void *o, hipStream_t stream);

// Prefill plan: how a sequence is cut into segments and chunks.
struct PrefillPlan {
    int chunk;               // C
    int segments;            // P >= 1
    int64_t segment_tokens;  // tokens per segment (multiple of C), last segment may be shorter
    int pre_split;           // R in {1, 2}: the pre-pass and the scan work on R pieces per segment (every segment but the last)
    size_t state_elems;      // B*H*d_k*d_v
    size_t ws_state_bytes;   // one slot of both states (fp32) per (piece, sequence, head) when P > 1: R (P - 1) + 1 pieces
    size_t ws_decay_bytes;   // one slot of both decays (fp32 log2) per (piece, sequence, head) when P > 1
    int64_t max_items;       // packed sequences with P > 1: capacity of the list of all segments (else 0)
    int64_t max_pre_items;   //   and of the list of segments that have a successor
    size_t ws_lists_bytes;   //   and the bytes of the lists
    size_t ws_total_bytes;
};
bool prefill_plan(const dsla_desc &d, int64_t T, PrefillPlan *plan);  // false: unsupported combination
bool prefill_plan_varlen(const dsla_desc &d, int64_t total_T, int64_t max_T, PrefillPlan *plan);
// cu_seqlens == nullptr: B sequences of T tokens each; else packed sequences and T = upper bound of their lengths.
// seq_index (with cu_seqlens only): which packed sequences take part; nullptr: all, in order.
// state_slot == nullptr: sequence b owns entry b of S1, S2.
// ext (or nullptr): a launch for one pair of states of a layer with N states: explicit blend coefficients, key/value
// heads shared by groups of query heads, and the result added to what o holds.
struct PrefillExt {
    int Hkv;
    int accumulate;
    int beta;   // nonzero: one state with the outer-product gate (g1 = log alpha, g2 = log beta, S1 only, wa only)
    float wa, wb;
    const float *wa_per_head, *wb_per_head;   // optional device arrays [H]
};
hipError_t launch_prefill(const dsla_desc &d, const PrefillPlan &plan, int64_t T, const int32_t *cu_seqlens,
                          const int32_t *seq_index, const int32_t *state_slot, const void *q, const void *k, const void *v, const void *g1,
                          const void *g2, float *S1, float *S2, void *o, void *workspace, hipStream_t stream,
                          const PrefillExt *ext = nullptr);

// Single-query attention kernels (entropy of the final query, decode attention over a cache): the keys of one
// (batch, head) are split into `parts` ranges, each leaving a record of floats_per_part floats to merge.
struct EntropyPlan {
    int parts;
    int64_t rows_per_part;
    size_t ws_bytes;   // parts > 1: one record per (batch, head, part)
};
bool entropy_plan(int B, int H, int d, int64_t T, EntropyPlan *plan, int floats_per_part = 3);  // false: head size not built
hipError_t launch_attn_decode(int B, int H, int d, int64_t T, int io_dtype, const EntropyPlan &plan, float scale,
                              const void *q_last, const void *k, const void *v, const int32_t *seq_lens, void *o,
                              void *workspace, hipStream_t stream);
hipError_t launch_project(int64_t M, int K, int n_out, int width, const void *x, const void *w, const float *bias,
                          void *const *outs, hipStream_t stream);
hipError_t launch_attn_prefill(int B, int H, int d, int64_t T, float scale, const void *q, const void *k, const void *v,
                               void *o, hipStream_t stream);
hipError_t launch_entropy(int B, int H, int d, int64_t T, int io_dtype, const EntropyPlan &plan, float scale,
                          const void *q_last, const void *k, float *entropy, void *workspace, hipStream_t stream);

}  // namespace dsla
