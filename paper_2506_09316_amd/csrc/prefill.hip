// Chunked DSLA prefill for gfx950 (paper Section 4.1: state-update equation and blended
// read-out, evaluated 32 tokens at a time).
//
// The token recurrence is regrouped so that every bracket is a dense contraction and runs on MFMA; the
// algebra is written out above the kernel body ("Chunk algebra").  With Qc = [Q~^1 | Q~^2] and
// Kc = [K~^1 | K~^2] (width 2 d_k) the blend of the two states is part of the contractions:
// scores = Qc Kc^T, carried read-out = Qc [T^1; T^2].
//
// Parallel decomposition.  A sequence is cut into P segments so that B*H*P workgroups fill the
// chip.  (1) segment_state: every segment but the last computes, from a zero state, its state
// contribution U and its total log-decay.  (2) segment_scan: an elementwise scan over segments
// turns these into the true state entering each segment.  (3) chunk_loop: every segment runs the
// fused step loop from its true initial state and writes o; the last segment writes the final
// states.  P = 1 runs (3) alone.  (1) and (3) are one kernel template; for 16-bit inputs and gates at d = 128, (1) has a
// kernel of its own that walks a segment backwards (segment_state_fast_kernel, below the template).
// Packed sequences of different lengths share one segment length; a one-workgroup kernel (segment_list) turns
// their offsets into the lists of (sequence, segment) pairs that (1) and (3) take their work from, so that no
// workgroup is launched for a segment that does not exist.  Sequences may be a subset of the packed batch and
// their states entries of a pool (both through index arrays).  Gates arrive as log-gates or as the
// pre-activations of a temperature-sigmoid, which the producers then apply themselves.
//
// Workgroup = D/8 wavefronts (D = d_k = d_v): D/32 consumers and D/32 producers, see "Workgroup layout".
// Consumer w owns state columns [32w, 32w+32) of both states for all d_k rows, as fp32 MFMA accumulators
// (tiles with m = state row, n = column).  Because an MFMA accumulator tile and an MFMA input fragment both
// index lanes by the tile column, those accumulators are fed back as the input fragment of the carried
// read-out without passing through LDS; the partner operand is stored in LDS with the matching order of
// the contraction index (bits 2 and 3 of the feature index swapped).
#include <cstdio>
#include <type_traits>
#include <utility>

#include "dsla_internal.h"

namespace dsla {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for the global
// loads of the next chunk that are deliberately left in flight across the contraction phases.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_sched_barrier(0);   // phases are not interleaved by the instruction scheduler
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------------------------
// LDS access by byte address.  Every LDS address below is "per-lane base register + compile-time
// constant"; the bases are computed once and passed through opaque() so that the compiler keeps them
// as they are instead of materialising one register per (base, constant) pair.
// ---------------------------------------------------------------------------------------------
#define DSLA_LDS __attribute__((address_space(3)))
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((DSLA_LDS const char *)p));
}
__device__ __forceinline__ uint32_t opaque(uint32_t x)
{
    asm volatile("" : "+v"(x));
    return x;
}
template <class T>
struct LdsPtr {
    typedef T DSLA_LDS *type;   // pointer into LDS (32-bit)
};
template <class T>
__device__ __forceinline__ T lds_ld(uint32_t a)
{
    return *reinterpret_cast<typename LdsPtr<const T>::type>(static_cast<uintptr_t>(a));
}
template <class T>
__device__ __forceinline__ void lds_st(uint32_t a, T v)
{
    *reinterpret_cast<typename LdsPtr<T>::type>(static_cast<uintptr_t>(a)) = v;
}

// ---------------------------------------------------------------------------------------------
// Arithmetic-type policies: how a contraction operand is stored in LDS and fed to MFMA.
// A "fragment" is the 8 contraction-index values one lane supplies for a block of 16 contraction
// indices (lane group g = lane/32 supplies indices 8g..8g+7 of the block).
// ---------------------------------------------------------------------------------------------
struct ArithBf16 {
    static constexpr int ESZ = 2;  // bytes per LDS element
    struct Frag {
        bf16x8 v;
    };
    struct Row8 {   // 8 operand values of one token, packed
        u32x4 u;
    };
    static __device__ __forceinline__ Frag load_frag(uint32_t a)
    {
        Frag f;
        f.v = __builtin_bit_cast(bf16x8, lds_ld<u32x4>(a));
        return f;
    }
    // Two transposing 8-byte reads (see Kern::consume): contraction positions 0..3 from address a, 4..7 from a + step.
    static __device__ __forceinline__ Frag load_frag_tr(uint32_t a, uint32_t step)
    {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4 DSLA_LDS *>(static_cast<uintptr_t>(a)));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4 DSLA_LDS *>(static_cast<uintptr_t>(a + step)));
        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
        Frag f;
        f.v = __builtin_bit_cast(bf16x8, u32x4{l2[0], l2[1], h2[0], h2[1]});
        return f;
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        f32x2 x = {a, b};
        bf16x2 y = __builtin_convertvector(x, bf16x2);
        return __builtin_bit_cast(uint32_t, y);
    }
    static __device__ __forceinline__ Row8 pack_row(const float (&x)[8])
    {
        Row8 r;
        r.u = u32x4{pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7])};
        return r;
    }
    static __device__ __forceinline__ void store_row(uint32_t a, const Row8 &r) { lds_st<u32x4>(a, r.u); }
    static constexpr uint32_t kSignBits = 0x80008000u;   // sign bits of the two values of a packed word
    static __device__ __forceinline__ Row8 flip_sign(Row8 r, uint32_t bits)   // bits: kSignBits or 0
    {
        r.u ^= u32x4{bits, bits, bits, bits};
        return r;
    }
    // element e of RPT consecutive tokens -> RPT adjacent LDS elements
    template <int RPT>
    static __device__ __forceinline__ void store_tokens(uint32_t a, const Row8 (&r)[RPT], int e)
    {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        const uint32_t lo = __builtin_amdgcn_perm(r[1].u[e >> 1], r[0].u[e >> 1], sel);
        if constexpr (RPT == 4) {
            const uint32_t hi = __builtin_amdgcn_perm(r[3].u[e >> 1], r[2].u[e >> 1], sel);
            lds_st<u32x2>(a, u32x2{lo, hi});
        } else {
            lds_st<uint32_t>(a, lo);
        }
    }
    static __device__ __forceinline__ void store4(uint32_t a, float x0, float x1, float x2, float x3)
    {
        lds_st<u32x2>(a, u32x2{pack2(x0, x1), pack2(x2, x3)});
    }
    static __device__ __forceinline__ f32x4 load4(uint32_t a)   // four adjacent operand elements
    {
        const u32x2 u = lds_ld<u32x2>(a);
        return f32x4{__uint_as_float(u[0] << 16), __uint_as_float(u[0] & 0xffff0000u), __uint_as_float(u[1] << 16),
                     __uint_as_float(u[1] & 0xffff0000u)};
    }
    static __device__ __forceinline__ Frag from_acc(const f32x16 &acc, int half)
    {
        const u32x4 u = {pack2(acc[8 * half + 0], acc[8 * half + 1]), pack2(acc[8 * half + 2], acc[8 * half + 3]),
                         pack2(acc[8 * half + 4], acc[8 * half + 5]), pack2(acc[8 * half + 6], acc[8 * half + 7])};
        Frag f;
        f.v = __builtin_bit_cast(bf16x8, u);
        return f;
    }
    static __device__ __forceinline__ void mma(f32x16 &acc, const Frag &a, const Frag &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
    }
};

struct ArithF32 {
    static constexpr int ESZ = 4;
    struct Frag {
        float v[8];
    };
    struct Row8 {
        float x[8];
    };
    static __device__ __forceinline__ Frag load_frag(uint32_t a)
    {
        const f32x4 lo = lds_ld<f32x4>(a), hi = lds_ld<f32x4>(a + 16);
        Frag f;
        f.v[0] = lo[0]; f.v[1] = lo[1]; f.v[2] = lo[2]; f.v[3] = lo[3];
        f.v[4] = hi[0]; f.v[5] = hi[1]; f.v[6] = hi[2]; f.v[7] = hi[3];
        return f;
    }
    static __device__ __forceinline__ Frag load_frag_tr(uint32_t, uint32_t) { return Frag{}; }   // 16-bit storage only
    static __device__ __forceinline__ Row8 pack_row(const float (&x)[8])
    {
        Row8 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r.x[e] = x[e];
        return r;
    }
    static __device__ __forceinline__ void store_row(uint32_t a, const Row8 &r)
    {
        lds_st<f32x4>(a, f32x4{r.x[0], r.x[1], r.x[2], r.x[3]});
        lds_st<f32x4>(a + 16, f32x4{r.x[4], r.x[5], r.x[6], r.x[7]});
    }
    static constexpr uint32_t kSignBits = 0x80000000u;
    static __device__ __forceinline__ Row8 flip_sign(Row8 r, uint32_t bits)   // bits: kSignBits or 0
    {
#pragma unroll
        for (int e = 0; e < 8; ++e) r.x[e] = __uint_as_float(__float_as_uint(r.x[e]) ^ bits);
        return r;
    }
    template <int RPT>
    static __device__ __forceinline__ void store_tokens(uint32_t a, const Row8 (&r)[RPT], int e)
    {
        if constexpr (RPT == 4)
            lds_st<f32x4>(a, f32x4{r[0].x[e], r[1].x[e], r[2].x[e], r[3].x[e]});
        else
            lds_st<f32x2>(a, f32x2{r[0].x[e], r[1].x[e]});
    }
    static __device__ __forceinline__ void store4(uint32_t a, float x0, float x1, float x2, float x3)
    {
        lds_st<f32x4>(a, f32x4{x0, x1, x2, x3});
    }
    static __device__ __forceinline__ f32x4 load4(uint32_t a) { return lds_ld<f32x4>(a); }
    static __device__ __forceinline__ Frag from_acc(const f32x16 &acc, int half)
    {
        Frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f.v[e] = acc[8 * half + e];
        return f;
    }
    // 32x32x2 fp32 MFMA: lane group g supplies one contraction index per instruction.
    static __device__ __forceinline__ void mma(f32x16 &acc, const Frag &a, const Frag &b)
    {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[e], b.v[e], acc, 0, 0, 0);
    }
};

template <class TIO>
using ArithOf = typename std::conditional<std::is_same<TIO, bf16_t>::value, ArithBf16, ArithF32>::type;

// ---- raw global loads (kept unconverted while in flight); address = uniform base + 32-bit lane offset ----
template <class T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
    u32x4 u;
    __device__ __forceinline__ void load(const bf16_t *base, uint32_t elem_off)
    {
        u = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(base) + elem_off * 2u);
    }
    __device__ __forceinline__ void zero() { u = u32x4{0, 0, 0, 0}; }
    __device__ __forceinline__ void fill_huge() { u = u32x4{0x7e007e00u, 0x7e007e00u, 0x7e007e00u, 0x7e007e00u}; }   // 2^125
    // orders every later use of the loaded value after `dep` has been computed (no instruction is emitted)
    __device__ __forceinline__ void pin_after(float dep) { asm volatile("" : "+v"(u) : "v"(dep)); }
    __device__ __forceinline__ void unpack(float (&f)[8]) const
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            f[2 * w] = __uint_as_float(u[w] << 16);
            f[2 * w + 1] = __uint_as_float(u[w] & 0xffff0000u);
        }
    }
};
template <>
struct Raw8<float> {
    f32x4 a, b;
    __device__ __forceinline__ void load(const float *base, uint32_t elem_off)
    {
        const char *p = reinterpret_cast<const char *>(base) + elem_off * 4u;
        a = *reinterpret_cast<const f32x4 *>(p);
        b = *reinterpret_cast<const f32x4 *>(p + 16);
    }
    __device__ __forceinline__ void zero() { a = b = f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ __forceinline__ void fill_huge() { a = b = f32x4{0x1p125f, 0x1p125f, 0x1p125f, 0x1p125f}; }
    __device__ __forceinline__ void pin_after(float dep) { asm volatile("" : "+v"(a), "+v"(b) : "v"(dep)); }
    __device__ __forceinline__ void unpack(float (&f)[8]) const
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            f[w] = a[w];
            f[4 + w] = b[w];
        }
    }
};
template <class T>
struct Raw4;
template <>
struct Raw4<bf16_t> {
    u32x2 u;
    __device__ __forceinline__ void load(const bf16_t *base, uint32_t elem_off)
    {
        u = *reinterpret_cast<const u32x2 *>(reinterpret_cast<const char *>(base) + elem_off * 2u);
    }
    __device__ __forceinline__ void zero() { u = u32x2{0, 0}; }
};
template <>
struct Raw4<float> {
    f32x4 a;
    __device__ __forceinline__ void load(const float *base, uint32_t elem_off)
    {
        a = *reinterpret_cast<const f32x4 *>(reinterpret_cast<const char *>(base) + elem_off * 4u);
    }
    __device__ __forceinline__ void zero() { a = f32x4{0.f, 0.f, 0.f, 0.f}; }
};

// Transposed store of V: element e (0..3) of RPT consecutive tokens -> RPT adjacent LDS elements.
// bf16 data is moved with byte permutes (no conversion); fp32 data is stored as is.
template <int RPT>
__device__ __forceinline__ void store_v_tokens(uint32_t a, const Raw4<bf16_t> (&v)[RPT], int e)
{
    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
    const uint32_t lo = __builtin_amdgcn_perm(v[1].u[e >> 1], v[0].u[e >> 1], sel);
    if constexpr (RPT == 4) {
        const uint32_t hi = __builtin_amdgcn_perm(v[3].u[e >> 1], v[2].u[e >> 1], sel);
        lds_st<u32x2>(a, u32x2{lo, hi});
    } else {
        lds_st<uint32_t>(a, lo);
    }
}
template <int RPT>
__device__ __forceinline__ void store_v_tokens(uint32_t a, const Raw4<float> (&v)[RPT], int e)
{
    if constexpr (RPT == 4)
        lds_st<f32x4>(a, f32x4{v[0].a[e], v[1].a[e], v[2].a[e], v[3].a[e]});
    else
        lds_st<f32x2>(a, f32x2{v[0].a[e], v[1].a[e]});
}

template <int RPT>
__device__ __forceinline__ void store_v_tokens(uint32_t a, const Raw8<bf16_t> (&v)[RPT], int e)
{
    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
    const uint32_t lo = __builtin_amdgcn_perm(v[1].u[e >> 1], v[0].u[e >> 1], sel);
    if constexpr (RPT == 4) {
        const uint32_t hi = __builtin_amdgcn_perm(v[3].u[e >> 1], v[2].u[e >> 1], sel);
        lds_st<u32x2>(a, u32x2{lo, hi});
    } else {
        lds_st<uint32_t>(a, lo);
    }
}
template <int RPT>
__device__ __forceinline__ void store_v_tokens(uint32_t a, const Raw8<float> (&v)[RPT], int e)
{
    auto pick = [&](const Raw8<float> &r) -> float { return e < 4 ? r.a[e & 3] : r.b[e & 3]; };
    if constexpr (RPT == 4)
        lds_st<f32x4>(a, f32x4{pick(v[0]), pick(v[1]), pick(v[2]), pick(v[3])});
    else
        lds_st<f32x2>(a, f32x2{pick(v[0]), pick(v[1])});
}

// a loaded row piece of V as it is (16-bit storage only)
__device__ __forceinline__ void store_v_row(uint32_t a, const Raw8<bf16_t> &v) { lds_st<u32x4>(a, v.u); }

// four adjacent output elements -> global
__device__ __forceinline__ void store4_global(bf16_t *p, float a, float b, float c, float d)
{
    *reinterpret_cast<u32x2 *>(p) = u32x2{ArithBf16::pack2(a, b), ArithBf16::pack2(c, d)};
}
__device__ __forceinline__ void store4_global(float *p, float a, float b, float c, float d)
{
    *reinterpret_cast<f32x4 *>(p) = f32x4{a, b, c, d};
}

// Software-pipelined sequence of N steps: the LDS fragment of step s + DEPTH is requested before the
// MFMA of step s is issued, so that LDS latency overlaps DEPTH matrix instructions.  Fully unrolled.
// kTr: the fragments come from rows by two transposing reads, the second TR_STEP bytes (two row slots) further.
template <int N, int DEPTH, class ARITH, bool kTr = false, class AddrF, class StepF>
__device__ __forceinline__ void pipelined_steps(AddrF addr, StepF step, uint32_t tr_step = 0)
{
    auto load = [&](int i) { return kTr ? ARITH::load_frag_tr(addr(i), tr_step) : ARITH::load_frag(addr(i)); };
    typename ARITH::Frag buf[DEPTH];
#pragma unroll
    for (int i = 0; i < DEPTH && i < N; ++i) buf[i] = load(i);
#pragma unroll
    for (int s = 0; s < N; ++s) {
        const typename ARITH::Frag cur = buf[s % DEPTH];
        if (s + DEPTH < N) buf[s % DEPTH] = load(s + DEPTH);
        step(s, cur);
    }
}

// ---------------------------------------------------------------------------------------------
struct PrefillArgs {
    const void *q, *k, *v, *g1, *g2;
    void *o;
    float *S1, *S2;          // caller's states
    // One workspace slot per (segment, sequence, head): slot = (p B + b) H + h, or with work lists
    // (seg_first[b] + p) H + h.  The last segment of a sequence has no decay entry that anyone reads.
    float *ws_state;         // [slot][2][D][D] fp32 (P > 1): state at the start of the segment
    float *ws_decay;         // [slot][2][D] fp32 (P > 1): log2 of the decay over the segment
    const float *gamma_per_head;
    const int32_t *cu;       // packed sequences: [B + 1] token offsets (sequence b = tokens cu[b] .. cu[b+1]-1); or null
    const int32_t *seq;      // with cu: [B] which of the packed sequences take part (entry b names sequence seq[b]); or null (all, in order)
    const int32_t *slot;     // [B] index of each sequence's states in S1, S2; or null (sequence b uses entry b)
    // Packed sequences cut into segments: the work lists written by segment_list_kernel.  A workgroup is
    // (list entry, head); entries past the count exit.  Null when every sequence is one segment or cu is null.
    const int32_t *seg_first;   // [B + 1] index of the first segment of each sequence among all segments
    const int32_t *seg_count;   // [2] entries in list_full, list_pre
    const int2 *list_full;      // (sequence, segment) of every segment
    const int2 *list_pre;       // (sequence, segment) of every segment that is followed by another one
    int64_t T;               // tokens per sequence (cu == null); with cu: upper bound of the sequence lengths
    int64_t seg_tokens;
    int H;
    int P;
    int zero_init;           // nonzero: the states are zero on entry (the caller's S1, S2 are only written)
    int32_t *status;         // optional device word: set to DSLA_STATUS_GATE_DOMAIN by a step whose gates leave the domain
    float gamma, scale;
    // Extended launches (Kern<.., kExt = true>): explicit blend coefficients of the two states instead of
    // (gamma, 1 - gamma), key/value heads shared by groups of query heads, and output added to what o holds.
    int Hkv;                 // key/value heads (k, v are [..][Hkv][D]); == H in ordinary launches
    int explicit_w;          // nonzero: the blend coefficients are wa, wb (or the per-head arrays)
    int accumulate;          // nonzero: o += result instead of o = result
    int beta;                // nonzero (Kern<.., kBeta = true>): one state with the outer-product gate, see "Beta mode"
    float wa, wb;
    const float *wa_per_head, *wb_per_head;   // optional [H]
    float gate_inv_tau;      // 0: g1, g2 are log-gates; else they are pre-activations and this is 1 / tau
    int slot_mul;            // chunk loop: segment p starts from workspace slot p * slot_mul (the pre-pass and the scan may
                             // work on pieces of a segment: see PrefillPlan::pre_split)
};

// Workgroup layout: producer / consumer wavefronts.  4 D threads = D/8 wavefronts.  The first D/32
// wavefronts are CONSUMERS: wavefront ct owns columns [32 ct, 32 ct + 32) of BOTH states for all d_k rows as fp32
// MFMA accumulators and runs every contraction of a step.  The other D/32 wavefronts are PRODUCERS: they load
// the inputs of later steps, run the gate scan and write the contraction operands of the NEXT step into the
// other half of a double-buffered LDS.  One workgroup barrier per step hands a finished operand set from the
// producers to the consumers.  Each SIMD hosts one consumer and one producer wavefront, so the VALU-bound
// preparation and the MFMA-bound contractions of neighbouring steps overlap.  A step is S = 32 tokens (a chunk
// of 64 is two steps): two operand sets of 32 tokens fit in the 160 KB LDS, two sets of 64 do not.
//
// Step algebra (Section 4.1 unrolled over the S = 32 tokens of a step).  Per state and feature: b_s = log2 of the gate
// product from the first token of the step up to and including token s (b_s <= 0), R = -b_31 the log2 decay of the whole
// step, and c_s = b_s + R/2 the same exponent centred on the step, so that |c_s| <= R/2.  T = the state in the frame of
// the middle of the step, T = 2^{-R/2} S at the start of the step:
//     Q~ = gamma_i scale q 2^{c}             K~ = k 2^{-c}                 (factors between 2^{-R/2} and 2^{+R/2})
//     o  =  Q~ T  +  mask_{key <= query}(Q~ K~^T) V                        (both states in one contraction of width 2 d_k)
//     T <-  T + K~^T V
//   between two steps the state moves from one middle frame to the next, at the end of a segment to its own frame:
//     T <-  diag(2^{-(R + R_next)/2}) T          (R_next = 0 after the last step)
// Centring halves the largest exponent a step can produce: the factors stay finite while R < 2 * 115, and nothing
// links the exponents of different steps.
//
// Beta mode (Kern<.., kBeta = true>, extended launches only): ONE state with the outer-product gate alpha^T beta of the
// background section on gated linear attention, S[d][j] <- alpha[d] beta[j] S[d][j] + k[d] v[j].  The tensor g1 holds
// log alpha as usual, g2 holds log beta (one value per token and COLUMN), S1 is the state, S2 is not used.  The decay
// along the columns is split like the one along the rows: with c' the centred cumulative log2 beta of a step,
//     V~ = v 2^{-c'}        o = 2^{+c'} . (Q~ T + mask(Q~ K~^T) V~)        T <- T + K~^T V~
// and T lives in the middle frame of the step for rows and columns alike.  The machinery of the second state carries
// beta: its gate scan gives c', its Q~ slot in LDS holds the output factors 2^{c'}, its slot of frame changes those of
// the columns; its K~ and its half of the contractions do not exist.
template <int D, class TIO, class TG, bool kFull, bool kExt = false, bool kBeta = false>
struct Kern {
    static_assert(kExt || !kBeta, "beta mode is an extended launch");
    static constexpr int NST = kBeta ? 1 : 2;   // states in the contractions
    using A = ArithOf<TIO>;
    using Frag = typename A::Frag;
    using Row8 = typename A::Row8;
    static constexpr int ESZ = A::ESZ;

    static constexpr int S = 32;            // tokens per step
    static constexpr int CT = D / 32;       // column tiles = consumer wavefronts = producer wavefronts
    static constexpr int NW = 2 * CT;       // wavefronts
    static constexpr int NT = 64 * NW;      // threads (= 4 D)
    static constexpr int SGN = 16;          // token pairs per step
    static constexpr int RPT = 2;           // tokens per producer thread
    static constexpr int QP = 2 * D + 8;    // pitch of row-layout operands (elements)
    // Token-contiguous operands (Kt, Vt): a row holds the S tokens of one feature (column) as 4 pieces of 8 tokens,
    // without padding; piece c of row R sits at piece position c ^ ((R / 2) % 4), so that the 8 rows a group of 8
    // lanes reads with one 16-byte access each fall into 8 different bank groups.
    static constexpr int TP = S;            // pitch of token-contiguous operands (elements)
    static __device__ __forceinline__ uint32_t tpiece(uint32_t piece, uint32_t row) { return piece ^ ((row >> 1) & 3u); }
    static constexpr int DT = D / 32;       // 32-row tiles of a state
    static constexpr int KB = S / 16;       // contraction blocks over tokens
    static constexpr int NK = 2 * D / 16;   // contraction blocks over the 2 d_k features

    // LDS map (bytes).  Two operand sets; per set:
    static constexpr uint32_t O_QS = 0;                                        // [token][i*D + d]            Q'
    // K~: 16-bit storage keeps ONE copy, in rows [token][i*D + d] of pitch QP; the consumers read it as rows (scores)
    // and, for the update, transposed with ds_read_b64_tr_b16.  Token t sits in row slot kslot(t): the two low bit pairs
    // of the token index swapped.  The 16 rows that 16 lanes read at the same feature then lie in 16 different slots
    // (each slot shifts the banks by 16 bytes: pitch), and the 4 consecutive tokens a pass of the transposing read
    // takes 64 bytes each from lie 4 slots apart: 64 bytes apart in the banks.  32-bit storage keeps two copies: rows
    // (step loop only) and the token-contiguous one [i*D + rho(d)][rho(token)].
    // (Step loop only: in the segment pre-pass, whose consumers have little else to do, the doubled number of LDS read
    // instructions gets in the way of the producers' gate scan, which is bound by its LDS round trips: 119.6 against
    // 116.8 us.)
    static constexpr bool kTrK = ESZ == 2 && kFull;
    static __device__ __forceinline__ uint32_t kslot(uint32_t t) { return (t & ~15u) | ((t & 3u) << 2) | ((t >> 2) & 3u); }
    static constexpr uint32_t O_KS = O_QS + (kFull ? S * QP * ESZ : 0);
    static constexpr uint32_t O_KT = O_KS + ((kFull || kTrK) ? S * QP * ESZ : 0);
    // V: 16-bit storage keeps the rows as loaded, [token][column] without padding, the 64-byte quarter q of row r at
    // quarter position q ^ vswz(r), and the consumers read them with the transposing LDS read, a pass of which takes one
    // quarter from each of 4 consecutive rows: they fall into different banks.  32-bit storage keeps the
    // token-contiguous copy [column][rho(token)].  Both take S * D elements.
    static constexpr bool kTrV = ESZ == 2;
    static __device__ __forceinline__ uint32_t vswz(uint32_t row) { return D == 128 ? (row & 3u) : ((row >> 1) & 1u); }
    static constexpr uint32_t O_VT = O_KT + (kTrK ? 0 : 2 * D * TP * ESZ);
    static constexpr uint32_t O_DEC = O_VT + D * TP * ESZ;                     // float [2D]  frame change after the step
    static constexpr uint32_t SET_BYTES = O_DEC + 2 * D * 4;
    static constexpr uint32_t LDS_MAX = 160 * 1024;                            // LDS of a gfx950 compute unit
    // Two operand sets where they fit (the producers then run a whole step ahead of the consumers); one set
    // otherwise (fp32 at d = 128): the producers then only load ahead and prepare between two barriers.
    static constexpr int SETS = (2 * SET_BYTES + CT * 4096 <= LDS_MAX) ? 2 : 1;
    static constexpr uint32_t O_CS = SETS * SET_BYTES;                         // per producer wavefront: float [2][16][32]
    // Output staging (16-bit io only): two buffers of S rows of d_v elements.  The consumers leave the output tile of
    // a step here and write it to memory one step later as whole rows (a row is then complete: it has passed the
    // barrier), which is what the memory system wants; 8-byte pieces straight from the accumulators cost a quarter
    // of the kernel time.
    static constexpr uint32_t O_ENT = O_CS + CT * 4096;                        // float [2D]  frame change into the first step
    static constexpr uint32_t LDS_NOSTAGE = O_ENT + 2 * D * 4, LDS_STAGE = LDS_NOSTAGE + 2 * S * D * ESZ;
    static constexpr bool kStage =   // only where it does not cost a resident workgroup
        kFull && ESZ == 2 && LDS_STAGE <= LDS_MAX && LDS_MAX / LDS_STAGE == LDS_MAX / LDS_NOSTAGE;
    static constexpr uint32_t O_ST = LDS_NOSTAGE;
    static constexpr uint32_t ST_BYTES = S * D * ESZ;
    static constexpr int NC = D * ESZ / 16;                                    // 16-byte pieces per output row
    static constexpr uint32_t LDS_BYTES = O_ST + (kStage ? 2 * ST_BYTES : 0);
    static_assert(LDS_BYTES <= LDS_MAX, "LDS budget");

    // rho: bits 2 and 3 of an index swapped.  Features are stored in Kt rows in rho order and tokens in Kt / Vt
    // columns in rho order.  With this order the 8 accumulator registers of one half of a 32x32 MFMA result tile
    // (lane group g holds tile rows 8a + 4g + b) are exactly the 8 contraction indices lane group g supplies in an
    // MFMA input fragment read from 8 consecutive positions, so results are fed back as inputs without LDS.
    static __device__ __forceinline__ uint32_t rho(uint32_t x) { return (x & ~12u) | ((x & 4u) << 1) | ((x & 8u) >> 1); }

    // Inputs of one step as loaded (unconverted): this thread's 2 tokens x 8 features.
    struct RawIO {
        Raw8<TIO> q[RPT], k[RPT], v[RPT];
    };
    struct RawGates {
        Raw8<TG> g1[RPT], g2[RPT];
    };
    // Where a producer lane reads a step from.  Loads are never predicated (the number of loads in flight stays
    // a compile-time fact, so waiting for the oldest never waits for the newest): a step past the end of the
    // segment re-reads the last one and a token past the end re-reads the last token; the producer zeroes those.
    struct StepSrc {
        const TIO *q, *k, *v;   // uniform: first token of the step, this (batch, head)
        const TG *g1, *g2;
        uint32_t off[RPT];      // per lane: element offset of token 2 sg + j, features 32 pw + 8 dgl ..
        uint32_t offkv[RPT];    // the same inside k and v when they have fewer heads (kExt only)
        __device__ __forceinline__ uint32_t kv(int j) const { return kExt ? offkv[j] : off[j]; }
    };
    static __device__ __forceinline__ void load_gates(RawGates &g, const StepSrc &s)
    {
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            g.g1[j].load(s.g1, s.off[j]);
            g.g2[j].load(s.g2, s.off[j]);
        }
    }
    static __device__ __forceinline__ void load_io(RawIO &r, const StepSrc &s)
    {
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            r.k[j].load(s.k, s.kv(j));
            if (kFull) r.q[j].load(s.q, s.off[j]);
            r.v[j].load(s.v, s.kv(j));
        }
    }
    // The loads a producer issues while it prepares step m, one at a time between its stages: q, k, v of step
    // m + 1 and the gates of step m + 3.  Slot numbers are constants after unrolling.
    struct NoLoads {
        __device__ __forceinline__ void at(int) const {}
    };
    struct NextLoads {
        RawIO &r;
        const StepSrc &rs;
        RawGates &g;
        const StepSrc &gs;
        __device__ __forceinline__ void at(int slot) const
        {
            if (slot == 0) g.g1[0].load(gs.g1, gs.off[0]);
            if (slot == 1) g.g1[1].load(gs.g1, gs.off[1]);
            if (slot == 2) g.g2[0].load(gs.g2, gs.off[0]);
            if (slot == 3) g.g2[1].load(gs.g2, gs.off[1]);
            if (slot == 4) r.k[0].load(rs.k, rs.kv(0));
            if (slot == 5) r.k[1].load(rs.k, rs.kv(1));
            if (slot == 6 && kFull) r.q[0].load(rs.q, rs.off[0]);
            if (slot == 7 && kFull) r.q[1].load(rs.q, rs.off[1]);
            if (slot == 8) r.v[0].load(rs.v, rs.kv(0));
            if (slot == 9) r.v[1].load(rs.v, rs.kv(1));
        }
    };

    // wavefront-private LDS hand-over: the LDS pipeline runs the requests of one wavefront in order; only the
    // compiler has to be kept from moving accesses across
    static __device__ __forceinline__ void wave_sync() { asm volatile("" ::: "memory"); }

    // Per-lane LDS addresses of a producer (operand set 0; a set adds SET_BYTES), computed once.
    // Lane (sg, dgl) of producer wavefront pw handles tokens 2sg, 2sg+1 and features 32 pw + 8 dgl .. + 7 of both
    // states (and the same columns of v); for the scan over tokens lane l owns column (state l/32, feature l%32).
    struct ProdAddr {
        uint32_t tot;   // scan scratch [state][sg][feature]: this lane's 8 features of state 0 (state 1: + 2048)
        uint32_t col;   // scan scratch: this lane's column, token pair 0
        uint32_t dec;   // decay factor of this lane's column
        uint32_t row;   // row-layout operands: token 2sg, element f0 (token + 1: + QP, state 1: + D elements)
        uint32_t kt[2];   // Kt: row of feature e = 0 of state 0, position of tokens 2sg, 2sg+1; [x]: for features e with (e/2)%2 = x
        uint32_t vt[4];   // Vt: row of column f0, position of tokens 2sg, 2sg+1; [x]: for columns e with (e/2)%4 = x
        uint32_t vrow[RPT];   // V rows (16-bit storage): token 2sg + j, this lane's 8 columns
        uint32_t krow[RPT];   // K~ rows (16-bit storage): row slot of token 2sg + j, element f0 (state 1: + D elements)
        uint32_t sg;
        uint32_t state;   // state of the column this lane scans
        bool preact;      // the gate tensors hold pre-activations, not log-gates (uniform)
        float unit;       // gate sums times this = log2 of the decay: log2 e for log-gates, 1 / tau for pre-activations
        __device__ __forceinline__ ProdAddr(uint32_t sm, int pw, uint32_t lane)
        {
            sg = lane >> 2;
            state = lane >> 5;
            const uint32_t dgl = lane & 3, f0 = 32 * pw + 8 * dgl;
            const uint32_t csw = sm + O_CS + pw * 4096;
            tot = csw + (sg * 32 + 8 * dgl) * 4;
            col = csw + ((lane >> 5) * SGN * 32 + (lane & 31)) * 4;
            dec = sm + O_DEC + ((lane >> 5) * D + 32 * pw + (lane & 31)) * 4;
            row = sm + (sg * RPT * QP + f0) * ESZ;
            // feature 8 dgl + e of the wavefront's 32 goes to row rho(8 dgl + e) = 16 (dgl/2) + 8 (e/4) + 4 (dgl%2) + e%4
            // the row of feature e is R = (multiple of 8) + 4 (dgl%2) + e%4 (+ 8 (e/4)): (R/2)%4 = 2 (dgl%2) + (e/2)%2
            const uint32_t tok = rho(2 * sg), piece = tok >> 3, within = tok & 7;
#pragma unroll
            for (uint32_t x = 0; x < 2; ++x)
                kt[x] = sm + O_KT + ((32 * pw + 16 * (dgl >> 1) + 4 * (dgl & 1)) * TP + 8 * (piece ^ (2 * (dgl & 1)) ^ x) + within) * ESZ;
            // the row of column e is R = 32 pw + 8 dgl + e: (R/2)%4 = (e/2)%4
#pragma unroll
            for (uint32_t x = 0; x < 4; ++x) vt[x] = sm + O_VT + (f0 * TP + 8 * (piece ^ x) + within) * ESZ;
#pragma unroll
            for (uint32_t j = 0; j < RPT; ++j) {
                const uint32_t r = sg * RPT + j;   // the lane's 8 columns are piece dgl of quarter pw of the row
                vrow[j] = sm + O_VT + r * (D * ESZ) + 64 * (static_cast<uint32_t>(pw) ^ vswz(r)) + 16 * dgl;
                krow[j] = sm + O_KS + (kslot(r) * QP + f0) * ESZ;
            }
        }
    };

    // ------------------------------------------------------------------------------------------------------
    // Producer, gate scan of one step, in three stages with a wavefront-private LDS round trip between them.  All 16
    // token pairs of a feature live in one wavefront, so the scan over the tokens needs no workgroup barrier.  The
    // stages of step m + 1 are spread over the operand preparation of step m, which hides the round trips.
    // ------------------------------------------------------------------------------------------------------
    struct ScanOut {
        float c[2][RPT][8];   // gate sums over this thread's tokens: c[i][j] = g[0] + .. + g[j]  (times ProdAddr::unit = log2 of a decay)
        float pre[2][8];      // gate sum from the first token of the chunk to before this thread's tokens
    };
    // Gate pre-activations z -> tau log2(alpha) for alpha = sigmoid(z)^(1/tau):
    //   tau log2 alpha = min(y, 0) - log2(1 + 2^-|y|),  y = z log2 e
    // (the 1 / tau is applied where the sums are exponentiated: ProdAddr::unit).
    static __device__ __forceinline__ void activate(float (&g)[8])
    {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float y = g[e] * kLog2e;
            const float l = __builtin_amdgcn_logf(1.0f + __builtin_amdgcn_exp2f(-__builtin_fabsf(y)));
            g[e] = fminf(y, 0.f) - l;
        }
    }
    // stage A: sums over this thread's tokens; totals of the token pair -> scan scratch.
    // `valid` = tokens of the step that exist; tokens past the end act as "no decay".
    static __device__ __forceinline__ void scan_a(const ProdAddr &pa, RawGates &r, int valid, ScanOut &o)
    {
        if (valid < S) {   // a token past the end: log-gate 0, or a pre-activation whose log-gate is exactly 0
#pragma unroll
            for (int j = 0; j < RPT; ++j)
                if (static_cast<int>(pa.sg) * RPT + j >= valid) {
                    if (pa.preact) {
                        r.g1[j].fill_huge();
                        r.g2[j].fill_huge();
                    } else {
                        r.g1[j].zero();
                        r.g2[j].zero();
                    }
                }
        }
        float g[8];
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            r.g1[j].unpack(g);
            if (pa.preact) activate(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) o.c[0][j][e] = j ? o.c[0][j - 1][e] + g[e] : g[e];
            r.g2[j].unpack(g);
            if (pa.preact) activate(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) o.c[1][j][e] = j ? o.c[1][j - 1][e] + g[e] : g[e];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t a = pa.tot + i * SGN * 32 * 4;
            lds_st<f32x4>(a, f32x4{o.c[i][RPT - 1][0], o.c[i][RPT - 1][1], o.c[i][RPT - 1][2], o.c[i][RPT - 1][3]});
            lds_st<f32x4>(a + 16, f32x4{o.c[i][RPT - 1][4], o.c[i][RPT - 1][5], o.c[i][RPT - 1][6], o.c[i][RPT - 1][7]});
        }
    }
    // stage B: scan of this lane's column over the 16 token pairs of the step, centred on the step: the exclusive
    // prefixes start at minus half of the step's gate sum, so that the exponents built from them span [-R/2, +R/2].
    // total: the gate sum of the column over the step (<= 0; times ProdAddr::unit = -R).
    static __device__ __forceinline__ void scan_b_read(const ProdAddr &pa, float (&t)[SGN])
    {
        wave_sync();
#pragma unroll
        for (int s2 = 0; s2 < SGN; ++s2) t[s2] = lds_ld<float>(pa.col + s2 * 32 * 4);
    }
    static __device__ __forceinline__ void scan_b(const ProdAddr &pa, const float (&t)[SGN], float &total)
    {
        float tot = (((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]))) +
                    (((t[8] + t[9]) + (t[10] + t[11])) + ((t[12] + t[13]) + (t[14] + t[15])));
        float run = -0.5f * tot;
#pragma unroll
        for (int s2 = 0; s2 < SGN; ++s2) {
            lds_st<float>(pa.col + s2 * 32 * 4, run);
            run += t[s2];
        }
        total = tot;
    }
    // The largest exponent a step may produce: Q~ and K~ carry 2^{+-R/2}, and bf16 / fp32 hold 2^{+-126}.
    static constexpr float kMaxStepLog2Decay = 230.f;
    // bookkeeping after stage B of a step: the segment's log2 decay, and the domain check
    static __device__ __forceinline__ void note_step(const ProdAddr &pa, float total, float &seg_log2_decay, int32_t *status)
    {
        const float r = total * pa.unit;   // -R
        seg_log2_decay += r;
        if (status && !(r >= -kMaxStepLog2Decay)) *status = DSLA_STATUS_GATE_DOMAIN;
    }
    // stage C: the exclusive prefixes of this thread's token pair
    static __device__ __forceinline__ void scan_c(const ProdAddr &pa, ScanOut &o)
    {
        wave_sync();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t a = pa.tot + i * SGN * 32 * 4;
            const f32x4 p0 = lds_ld<f32x4>(a), p1 = lds_ld<f32x4>(a + 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o.pre[i][e] = p0[e];
                o.pre[i][4 + e] = p1[e];
            }
        }
    }

    // ------------------------------------------------------------------------------------------------------
    // Producer, one call: operands of step m into operand set `set` from its inputs `r` and scan results `sc`, and,
    // interleaved, the gate scan of step m + 1 (gates `gn` -> `sn`) and the loads of later steps (`next`).
    // valid: of step m; valid_n: of step m + 1.  tot: in: gate sum of this lane's column over step m; out: over step
    // m + 1 (zero past the end of the segment).  The factor that takes the state from the middle frame of step m to
    // that of step m + 1 (to its own frame after the last step) goes into the operand set of step m.
    // ------------------------------------------------------------------------------------------------------
    template <class Loads>
    static __device__ __forceinline__ void produce(const ProdAddr &pa, uint32_t set, RawIO &r, const ScanOut &sc, int valid,
                                                   RawGates &gn, ScanOut &sn, int valid_n,
                                                   const float (&lg)[2], const uint32_t (&sgn)[2], float &tot,
                                                   float &seg_log2_decay, int32_t *status, const Loads &next)
    {
        const uint32_t so = set * SET_BYTES;
        if (valid < S) {   // ragged tail: tokens past the end act as "no key, no value"
#pragma unroll
            for (int j = 0; j < RPT; ++j)
                if (static_cast<int>(pa.sg) * RPT + j >= valid) {
                    r.k[j].zero();
                    r.v[j].zero();
                }
        }
        scan_a(pa, gn, valid_n, sn);
        next.at(0);
        next.at(1);

        Row8 kt[RPT];
        auto block = [&](int i, int j, int slot_k, int slot_q) {
            // K~ = k 2^{-c}, Q~ = gamma_i scale q 2^{c}: c = centred prefix before this thread's tokens + sum over its own
            next.at(slot_k);
            {   // row layout for the scores, token-contiguous (below) for the update
                float kf[8], kh[8];
                r.k[j].unpack(kf);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    kh[e] = kf[e] * __builtin_amdgcn_exp2f(-pa.unit * (sc.pre[i][e] + sc.c[i][j][e]));
                kt[j] = A::pack_row(kh);
                if constexpr (kTrK) A::store_row(pa.krow[j] + so + i * D * ESZ, kt[j]);
                else if (kFull) A::store_row(pa.row + so + O_KS + (j * QP + i * D) * ESZ, kt[j]);
            }
            next.at(slot_q);
            if (kFull) {
                float qf[8], qt[8];
                r.q[j].unpack(qf);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    qt[e] = qf[e] * __builtin_amdgcn_exp2f(fmaf(sc.pre[i][e] + sc.c[i][j][e], pa.unit, lg[i]));
                A::store_row(pa.row + so + O_QS + (j * QP + i * D) * ESZ, A::flip_sign(A::pack_row(qt), sgn[i]));
            }
        };
        auto kt_rows = [&](int i) {
            if constexpr (kTrK) return;   // the rows are the only copy
#pragma unroll
            for (int e = 0; e < 8; ++e)
                A::template store_tokens<RPT>(pa.kt[(e >> 1) & 1] + so + ((i * D + 8 * (e >> 2) + (e & 3)) * TP) * ESZ, kt, e);
        };

        // beta mode, tokens j: the scaled values V~ (kept for the token-contiguous copy) and the output factors
        Row8 vs[RPT];
        auto block_beta = [&](int j, int slot_a, int slot_b) {
            next.at(slot_a);
            float vf[8], vh[8], fo[8];
            r.v[j].unpack(vf);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float c = pa.unit * (sc.pre[1][e] + sc.c[1][j][e]);
                vh[e] = vf[e] * __builtin_amdgcn_exp2f(-c);
                fo[e] = __builtin_amdgcn_exp2f(c);
            }
            vs[j] = A::pack_row(vh);
            next.at(slot_b);
            if (kFull) A::store_row(pa.row + so + O_QS + (j * QP + D) * ESZ, A::pack_row(fo));
        };

        float t[SGN];
        scan_b_read(pa, t);   // the answers arrive while the first block is computed
        block(0, 0, 2, 3);
        {
            float tot_n;
            scan_b(pa, t, tot_n);
            lds_st<float>(pa.dec + so, __builtin_amdgcn_exp2f(0.5f * pa.unit * (tot + tot_n)));
            note_step(pa, tot_n, seg_log2_decay, status);
            tot = tot_n;
        }
        block(0, 1, 4, 5);
        kt_rows(0);
        scan_c(pa, sn);
        if constexpr (kBeta) {
            block_beta(0, 6, 7);
            block_beta(1, 8, 9);
            if constexpr (kTrV) {
#pragma unroll
                for (int j = 0; j < RPT; ++j) A::store_row(pa.vrow[j] + so, vs[j]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) A::template store_tokens<RPT>(pa.vt[(e >> 1) & 3] + so + e * TP * ESZ, vs, e);
            }
        } else {
            block(1, 0, 6, 7);
            block(1, 1, 8, 9);
            kt_rows(1);
            if constexpr (kTrV) {   // V as loaded
#pragma unroll
                for (int j = 0; j < RPT; ++j) store_v_row(pa.vrow[j] + so, r.v[j]);
            } else {                // V transposed
#pragma unroll
                for (int e = 0; e < 8; ++e) store_v_tokens<RPT>(pa.vt[(e >> 1) & 3] + so + e * TP * ESZ, r.v, e);
            }
        }
    }

    // ------------------------------------------------------------------------------------------------------
    // Producers that load whole 128-byte lines (kLineProd: 16-bit io, ordinary step loop).  The loads and stores of the
    // step loop alone, with no arithmetic, take as long as the whole kernel, and they take 5-7 % less when a load
    // instruction fetches pieces of 128 bytes instead of 64.  So here a producer wavefront prepares ONE state, 64 features
    // of it (one line of a row), all 32 tokens: a thread has 4 tokens x 8 features.  q and k are loaded by the wavefront
    // of either state (the second request hits in L2); v is split by tokens between them.  The gate scan stays inside
    // the wavefront: sums over the thread's 4 tokens, 8 totals per feature through wavefront-private LDS, one lane per
    // feature.  The operand sets, and with them the consumers, are the ones of the row producers above.
    // ------------------------------------------------------------------------------------------------------
    static constexpr bool kLineProd = ESZ == 2 && kFull && !kExt && !kBeta && SETS == 2;
    static constexpr int FHN = D / 64;   // lines per row = producer wavefronts per state
    static constexpr int TPT = 4;        // tokens per thread
    struct LineIO {
        Raw8<TIO> q[TPT], k[TPT], v[2];
    };
    struct LineGates {
        Raw8<TG> g[TPT];
    };
    struct LineSrc {
        const TIO *q, *k, *v;   // uniform: first token of the step, this (batch, head)
        const TG *g;            // the gates of this wavefront's state
        uint32_t off[TPT];      // per lane: element offset of token 4 sq + j, features 64 fh + 8 dg ..
        uint32_t offv[2];       // the same for this wavefront's share of v: token 16 st + 2 sq + j
    };
    struct LineNext {
        LineIO &r;
        const LineSrc &rs;
        LineGates &g;
        const LineSrc &gs;
        __device__ __forceinline__ void at(int slot) const
        {
            if (slot >= 0 && slot < 4) g.g[slot].load(gs.g, gs.off[slot]);
            if (slot >= 4 && slot < 8) r.k[slot - 4].load(rs.k, rs.off[slot - 4]);
            if (slot >= 8 && slot < 12) r.q[slot - 8].load(rs.q, rs.off[slot - 8]);
            if (slot == 12) r.v[0].load(rs.v, rs.offv[0]);
            if (slot == 13) r.v[1].load(rs.v, rs.offv[1]);
        }
    };
    struct LineAddr {
        uint32_t tot;         // scan scratch [8 quads][64 features] floats: this lane's 8 features of quad sq
        uint32_t col;         // scan scratch: this lane's column (feature lane of the 64), quad 0
        uint32_t dec;         // decay factor of this lane's column
        uint32_t qrow[TPT];   // Q~ row of token 4 sq + j, element st D + 64 fh + 8 dg
        uint32_t krow[TPT];   // K~: its row slot
        uint32_t vrow[2];     // V rows of token 16 st + 2 sq + j, columns 64 fh + 8 dg ..
        uint32_t sq, st, fh;
        bool preact;
        float unit;
        __device__ __forceinline__ LineAddr(uint32_t sm, int pw, uint32_t lane)
        {
            st = static_cast<uint32_t>(pw) / FHN;
            fh = static_cast<uint32_t>(pw) % FHN;
            sq = lane >> 3;
            const uint32_t dg = lane & 7, f0 = 64 * fh + 8 * dg;
            const uint32_t csw = sm + O_CS + pw * 4096;
            tot = csw + (sq * 64 + 8 * dg) * 4;
            col = csw + lane * 4;
            dec = sm + O_DEC + (st * D + 64 * fh + lane) * 4;
#pragma unroll
            for (uint32_t j = 0; j < TPT; ++j) {
                const uint32_t t = 4 * sq + j;
                qrow[j] = sm + O_QS + (t * QP + st * D + f0) * ESZ;
                krow[j] = sm + O_KS + (kslot(t) * QP + st * D + f0) * ESZ;
            }
#pragma unroll
            for (uint32_t j = 0; j < 2; ++j) {
                const uint32_t t = 16 * st + 2 * sq + j;
                vrow[j] = sm + O_VT + t * (D * ESZ) + 64 * ((f0 >> 5) ^ vswz(t)) + (f0 & 31u) * ESZ;
            }
        }
    };
    struct LineScan {
        float c[TPT][8];   // gate sums over this thread's tokens: c[j] = g[0] + .. + g[j]
        float pre[8];      // centred gate sum from the first token of the step to before this thread's tokens
    };
    static __device__ __forceinline__ void line_scan_a(const LineAddr &pa, LineGates &r, int valid, LineScan &o)
    {
        if (valid < S) {   // a token past the end: log-gate 0, or a pre-activation whose log-gate is exactly 0
#pragma unroll
            for (int j = 0; j < TPT; ++j)
                if (static_cast<int>(pa.sq) * TPT + j >= valid) {
                    if (pa.preact) r.g[j].fill_huge();
                    else r.g[j].zero();
                }
        }
        float g[8];
#pragma unroll
        for (int j = 0; j < TPT; ++j) {
            r.g[j].unpack(g);
            if (pa.preact) activate(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) o.c[j][e] = j ? o.c[j - 1][e] + g[e] : g[e];
        }
        lds_st<f32x4>(pa.tot, f32x4{o.c[TPT - 1][0], o.c[TPT - 1][1], o.c[TPT - 1][2], o.c[TPT - 1][3]});
        lds_st<f32x4>(pa.tot + 16, f32x4{o.c[TPT - 1][4], o.c[TPT - 1][5], o.c[TPT - 1][6], o.c[TPT - 1][7]});
    }
    static __device__ __forceinline__ void line_scan_b_read(const LineAddr &pa, float (&t)[8])
    {
        wave_sync();
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) t[s2] = lds_ld<float>(pa.col + s2 * 64 * 4);
    }
    static __device__ __forceinline__ void line_scan_b(const LineAddr &pa, const float (&t)[8], float &total)
    {
        const float tot = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        float run = -0.5f * tot;   // centred on the step, as scan_b
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) {
            lds_st<float>(pa.col + s2 * 64 * 4, run);
            run += t[s2];
        }
        total = tot;
    }
    static __device__ __forceinline__ void line_scan_c(const LineAddr &pa, LineScan &o)
    {
        wave_sync();
        const f32x4 p0 = lds_ld<f32x4>(pa.tot), p1 = lds_ld<f32x4>(pa.tot + 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o.pre[e] = p0[e];
            o.pre[4 + e] = p1[e];
        }
    }
    static __device__ __forceinline__ void line_note_step(const LineAddr &pa, float total, int32_t *status)
    {
        if (status && !(total * pa.unit >= -kMaxStepLog2Decay)) *status = DSLA_STATUS_GATE_DOMAIN;
    }
    // One call: operands of step m (state pa.st, 64 features) into operand set `set`, and, interleaved, the gate scan of
    // step m + 1 and the loads of later steps; as produce().  lg, sgn: of this wavefront's state.
    static __device__ __forceinline__ void line_produce(const LineAddr &pa, uint32_t set, LineIO &r, const LineScan &sc, int valid,
                                                        LineGates &gn, LineScan &sn, int valid_n, float lg, uint32_t sgn,
                                                        float &tot, int32_t *status, const LineNext &next)
    {
        const uint32_t so = set * SET_BYTES;
        if (valid < S) {   // ragged tail: tokens past the end act as "no key, no value"
#pragma unroll
            for (int j = 0; j < TPT; ++j)
                if (static_cast<int>(pa.sq) * TPT + j >= valid) r.k[j].zero();
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (static_cast<int>(16 * pa.st + 2 * pa.sq) + j >= valid) r.v[j].zero();
        }
        line_scan_a(pa, gn, valid_n, sn);
        next.at(0);
        next.at(1);
        next.at(2);
        next.at(3);
        auto block = [&](int j) {
            next.at(4 + j);
            float kf[8], kh[8];
            r.k[j].unpack(kf);
#pragma unroll
            for (int e = 0; e < 8; ++e) kh[e] = kf[e] * __builtin_amdgcn_exp2f(-pa.unit * (sc.pre[e] + sc.c[j][e]));
            A::store_row(pa.krow[j] + so, A::pack_row(kh));
            next.at(8 + j);
            float qf[8], qt[8];
            r.q[j].unpack(qf);
#pragma unroll
            for (int e = 0; e < 8; ++e) qt[e] = qf[e] * __builtin_amdgcn_exp2f(fmaf(sc.pre[e] + sc.c[j][e], pa.unit, lg));
            A::store_row(pa.qrow[j] + so, A::flip_sign(A::pack_row(qt), sgn));
        };
        float t[8];
        line_scan_b_read(pa, t);   // the answers arrive while the first block is computed
        block(0);
        {
            float tot_n;
            line_scan_b(pa, t, tot_n);
            lds_st<float>(pa.dec + so, __builtin_amdgcn_exp2f(0.5f * pa.unit * (tot + tot_n)));
            line_note_step(pa, tot_n, status);
            tot = tot_n;
        }
        block(1);
        line_scan_c(pa, sn);
        block(2);
        next.at(12);
        block(3);
        next.at(13);
#pragma unroll
        for (int j = 0; j < 2; ++j) store_v_row(pa.vrow[j] + so, r.v[j]);   // V as loaded
    }

    // ------------------------------------------------------------------------------------------------------
    // Consumer: all contractions of one step from operand set `set`.  acc[i][dt]: rows 32 dt .. of state i (Kt row
    // order), columns 32 ct ...  Register j of lane (ln, g) holds feature 32 dt + 16 (j / 8) + 8 g + j % 8.
    // Inside a chunk acc holds the state in the frame of the chunk start (see the step algebra above).
    // ------------------------------------------------------------------------------------------------------
    // Staged output rows of one step -> memory.  Consumer wavefront ct writes rows 32/CT * ct ..; a group of NC lanes
    // writes one whole row.
    static __device__ __forceinline__ void flush_rows(uint32_t sm, uint32_t parity, int ct, int lane, TIO *orow, uint32_t rs,
                                                      int valid, bool accumulate)
    {
        constexpr int RPI = 64 / NC;   // rows per instruction
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const uint32_t r = (S / CT) * ct + RPI * it + static_cast<uint32_t>(lane) / NC, c = static_cast<uint32_t>(lane) % NC;
            const uint32_t a = sm + O_ST + parity * ST_BYTES + r * (D * ESZ) + ((c ^ (r & (NC - 1))) << 4);
            u32x4 x = lds_ld<u32x4>(a);
            if (static_cast<int>(r) < valid) {
                u32x4 *dst = reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(orow) + (static_cast<size_t>(r) * rs * ESZ + c * 16));
                if (kExt && accumulate) {   // staged tiles are 16-bit: add to the eight values already there
                    const u32x4 old = *dst;
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        x[w] = ArithBf16::pack2(__uint_as_float(x[w] << 16) + __uint_as_float(old[w] << 16),
                                                __uint_as_float(x[w] & 0xffff0000u) + __uint_as_float(old[w] & 0xffff0000u));
                }
                // streaming store: the output is not read again by this call, and kept out of the caches it does not
                // delay the kernel that follows (measured: the next call's segment pre-pass 107 -> 95 us)
                __builtin_nontemporal_store(x, dst);
            }
        }
    }

    static __device__ __forceinline__ void consume(uint32_t sm, uint32_t set, f32x16 (&acc)[2][DT], int ct, int lane,
                                                   TIO *orow, uint32_t rs, int valid, uint32_t set_parity, bool accumulate)
    {
        const uint32_t lo = opaque(static_cast<uint32_t>(lane));
        const uint32_t ln = lo & 31, g = lo >> 5;
        const uint32_t setb = sm + set * SET_BYTES;
        // token block kb of a row: piece g + 2 kb, stored at piece position (g + 2 kb) ^ ((row / 2) % 4); all row
        // numbers used below are ln plus a multiple of 8
        const uint32_t p0 = 8 * tpiece(g, ln), p1 = 8 * tpiece(g + 2, ln);
        const uint32_t vt_r[KB] = {setb + O_VT + ((32 * ct + ln) * TP + p0) * ESZ, setb + O_VT + ((32 * ct + ln) * TP + p1) * ESZ};
        const uint32_t kt_r[KB] = {setb + O_KT + (ln * TP + p0) * ESZ, setb + O_KT + (ln * TP + p1) * ESZ};
        // transposing reads of the K~ rows (16-bit storage): lane l must end up with feature rho(l % 32) of a tile of 32
        // (the row order of the token-contiguous copy: the accumulators are fed back as fragments in it), so the lanes
        // that address piece s of 4 features point at piece (s swapped in its two bits); tokens as for V: row slots
        // 4 (l16 / 4) + g of a block of 16, and 2 slots further for the second read
        const uint32_t l16k = lo & 15, sgm = ((l16k & 1) << 1) | ((l16k >> 1) & 1);
        const uint32_t ktr_r = setb + O_KS + ((4 * (l16k >> 2) + g) * QP + 16 * ((lo >> 4) & 1) + 4 * sgm) * ESZ;
        const uint32_t dec_r = setb + O_DEC + (8 * g) * 4;

        // transposing reads of the V rows: the 16 lanes of a group address 4 tokens x 4 pieces of 4 columns and each
        // receives 4 tokens of ONE column; lane l ends up with column 32 ct + l % 32 and tokens 16 kb + 4 g + 0..3 (first
        // read) and 16 kb + 8 + 4 g + 0..3 (second read, 8 rows further): the order of the token-contiguous copies
        const uint32_t l16 = lo & 15, vr = 4 * g + (l16 >> 2);
        const uint32_t vs_r = setb + O_VT + vr * (D * ESZ) + 64 * (static_cast<uint32_t>(ct) ^ vswz(vr)) + 32 * ((lo >> 4) & 1) + 8 * (l16 & 3);
        Frag vf[KB];   // V fragments of this wavefront's columns: input of the output and of the update
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            if constexpr (kTrV) vf[kb] = A::load_frag_tr(vs_r + 16 * kb * (D * ESZ), 8 * (D * ESZ));
            else vf[kb] = A::load_frag(vt_r[kb]);
        }

        f32x16 oacc;
        if (kFull) {
            const uint32_t qs_r = setb + O_QS + (ln * QP + 8 * g) * ESZ;
            const uint32_t ks_r = setb + O_KS + ((kTrK ? kslot(ln) : ln) * QP + 8 * g) * ESZ;
            // One pass over the 2 d_k features, 16 at a time, with the Q~ fragment shared by two products:
            //   sc[j]   = S^T[key 8(j/4) + 4g + j%4][query ln]        (Q~ K~^T, both states blended)
            //   oacc[j] = o^T[column 8(j/4) + 4g + j%4][query ln]     (carried states: the accumulators themselves
            //                                                          are the input fragments)
            f32x16 sc;
#pragma unroll
            for (int j = 0; j < 16; ++j) sc[j] = oacc[j] = 0.f;
            {
                Frag held;   // the Ks fragment of a block waits here for its Qs partner
                pipelined_steps<NST * NK, 8, A>(
                    [&](int s2) -> uint32_t { return ((s2 & 1) ? qs_r : ks_r) + 16 * (s2 >> 1) * ESZ; },
                    [&](int s2, const Frag &f) {
                        if ((s2 & 1) == 0) {
                            held = f;
                        } else {
                            const int kb = s2 >> 1, i = kb / (2 * DT), dt = (kb / 2) % DT, half = kb & 1;
                            A::mma(sc, held, f);
                            A::mma(oacc, A::from_acc(acc[i][dt], half), f);
                        }
                    });
            }
            // keep key <= query; the two halves of the tile become the score fragments of the two token blocks
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t key = 8 * (j >> 2) + 4 * g + (j & 3);
                sc[j] = (key <= ln) ? sc[j] : 0.f;
            }
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) A::mma(oacc, vf[kb], A::from_acc(sc, kb));
        }
        __builtin_amdgcn_sched_barrier(0);   // the instruction groups requested below start here

        // ---- add K~^T V (the output tile finishes in the matrix pipeline meanwhile) ----
        {
            constexpr int NS = KB * NST * DT;   // (token block, state, tile)
            pipelined_steps<NS, 4, A, kTrK>(
                [&](int s2) -> uint32_t {
                    const int kb = s2 / (NST * DT), i = (s2 / DT) % NST, dt = s2 % DT;
                    if constexpr (kTrK) return ktr_r + (16 * kb * QP + i * D + 32 * dt) * ESZ;
                    else return kt_r[kb] + ((i * D + 32 * dt) * TP) * ESZ;
                },
                [&](int s2, const Frag &f) {
                    const int kb = s2 / (NST * DT), i = (s2 / DT) % NST, dt = s2 % DT;
                    A::mma(acc[i][dt], f, vf[kb]);
                },
                2 * QP * ESZ);
            constexpr int RD = ESZ == 2 ? 1 : 2, MM = ESZ == 2 ? 1 : 8;
            __builtin_amdgcn_sched_group_barrier(0x100, 4 * RD, 0);
#pragma unroll
            for (int s2 = 0; s2 < NS - 4; ++s2) {
                __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * MM, 0);
        }

        // ---- store: lane (ln, g) holds query ln, columns 32 ct + 8 jb + 4 g .. + 3 ----
        if constexpr (kBeta && kFull) {   // the output returns from the middle frame of the columns
            const uint32_t fo_r = setb + O_QS + (ln * QP + D + 32 * ct + 4 * g) * ESZ;
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                const f32x4 fo = A::load4(fo_r + 8 * jb * ESZ);
#pragma unroll
                for (int e = 0; e < 4; ++e) oacc[4 * jb + e] *= fo[e];
            }
        }
        if constexpr (kStage) {
            // piece (row ln, 16-byte piece c) lives at piece position c ^ (ln mod NC) of its row
            const uint32_t st_w = sm + O_ST + set_parity * ST_BYTES + ln * (D * ESZ) + 8 * g;
#pragma unroll
            for (int jb = 0; jb < 4; ++jb)
                A::store4(st_w + (((4 * ct + jb) ^ (ln & (NC - 1))) << 4), oacc[4 * jb], oacc[4 * jb + 1], oacc[4 * jb + 2],
                          oacc[4 * jb + 3]);
        } else if (kFull && static_cast<int>(ln) < valid) {
            TIO *op = orow + static_cast<size_t>(ln) * rs + 32 * ct + 4 * g;
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                float x0 = oacc[4 * jb], x1 = oacc[4 * jb + 1], x2 = oacc[4 * jb + 2], x3 = oacc[4 * jb + 3];
                if (kExt && accumulate) {
                    x0 += to_f32(op[8 * jb]);
                    x1 += to_f32(op[8 * jb + 1]);
                    x2 += to_f32(op[8 * jb + 2]);
                    x3 += to_f32(op[8 * jb + 3]);
                }
                store4_global(op + 8 * jb, x0, x1, x2, x3);
            }
        }

        // ---- the states move to the middle frame of the next step (after the last step: to their own frame) ----
        // (a block of its own for the register allocator: merged into the code above it costs four spilled registers)
        if (opaque(1u)) rescale(acc, dec_r, g, 32 * ct + ln);
    }

    // acc[i][dt][j] *= f[i D + feature of register j], f = 2 D floats at LDS address `fac` (+ 8 g floats for this lane);
    // beta mode: state 0 only, and every register of the lane also by the factor of the lane's column, f[D + column]
    // (`col` = the lane's column, 32 ct + ln).
    static __device__ __forceinline__ void rescale(f32x16 (&acc)[2][DT], uint32_t fac, uint32_t g, uint32_t col)
    {
        if constexpr (kBeta) {
            const float cf = lds_ld<float>(fac - 8 * g * 4 + (D + col) * 4);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[0][dt][j] *= cf;
        }
#pragma unroll
        for (int i = 0; i < NST; ++i) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                f32x4 dd[4];
#pragma unroll
                for (int jb = 0; jb < 4; ++jb)
                    dd[jb] = lds_ld<f32x4>(fac + (i * D + 32 * dt + 16 * (jb >> 1) + 4 * (jb & 1)) * 4);
#pragma unroll
                for (int jb = 0; jb < 4; ++jb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][dt][4 * jb + e] *= dd[jb][e];
            }
        }
    }

    static __device__ void run(const PrefillArgs &a, uint32_t sm)
    {
        const int tid = threadIdx.x;
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, kept in scalar registers

        int bidx, h, p;
        size_t slot0;   // workspace slot of (segment 0, this sequence, this head); segment p' is p' * slot_step further
        size_t slot_step;
        if (a.list_full) {
            const int it = blockIdx.x / a.H;
            if (it >= a.seg_count[kFull ? 0 : 1]) return;   // the lists are sized for the worst case
            const int2 e = (kFull ? a.list_full : a.list_pre)[it];
            bidx = e.x;
            p = e.y;
            h = blockIdx.x % a.H;
            slot0 = static_cast<size_t>(a.seg_first[bidx]) * a.H + h;
            slot_step = a.H;
        } else {
            const int nseg = kFull ? a.P : a.P - 1;
            const int bh = blockIdx.x / nseg;
            p = blockIdx.x % nseg;
            bidx = bh / a.H;
            h = bh % a.H;
            slot0 = bh;
            slot_step = gridDim.x / nseg;   // B H
        }

        // this sequence: first token in the token-major tensors, length, where its states live
        const int sq = (a.cu && a.seq) ? a.seq[bidx] : bidx;
        const int64_t seq0 = a.cu ? static_cast<int64_t>(a.cu[sq]) : static_cast<int64_t>(bidx) * a.T;
        const int64_t Tb = a.cu ? static_cast<int64_t>(a.cu[sq + 1]) - seq0 : a.T;
        const size_t sbh = static_cast<size_t>(a.slot ? a.slot[bidx] : bidx) * a.H + h;
        const int64_t t0 = static_cast<int64_t>(p) * a.seg_tokens;
        // A shorter sequence has fewer segments: the chunk loop has nothing to do past its end, and the state
        // of a segment is only needed if another segment follows.  (Uniform exit, before any barrier.)
        if (kFull ? t0 >= Tb : t0 + a.seg_tokens >= Tb) return;
        const int64_t t1 = (t0 + a.seg_tokens < Tb) ? t0 + a.seg_tokens : Tb;
        const int ntok = static_cast<int>(t1 - t0);               // tokens of this segment (>= 1)
        const int nsteps = (ntok + S - 1) / S;
        const uint32_t rs = static_cast<uint32_t>(a.H) * D;       // elements between consecutive tokens
        // uniform element offset of (b, t0, h, 0); per-lane offsets are 32-bit
        const size_t seg0 = (static_cast<size_t>(seq0 + t0) * a.H + h) * D;
        const size_t sstep = static_cast<size_t>(S) * rs;
        auto valid_of = [&](int n) -> int {   // tokens of step n that exist
            const int left = ntok - n * S;
            return left >= S ? S : (left > 0 ? left : 0);
        };
        // The step loop runs in pairs (set 0, set 1), so both roles pass the same number of barriers:
        // 1 + 2 * ceil(nsteps / 2) with two sets, twice as many in the loop with one.

        if (wave < CT) {
            // =============================== consumer ===============================
            const int ct = wave;
            const int ln = lane & 31, g = lane >> 5;
            f32x16 acc[2][DT];
            const uint32_t sbase = static_cast<uint32_t>(8 * g) * D + 32 * ct + ln;   // lane part of the state offset
            // A sequence that is cut into segments starts every segment, the first one included, from the slot the
            // segment scan filled: the workgroup of the last segment overwrites the caller's states in this same
            // launch, so no workgroup of such a sequence may read them here.  A sequence of one segment reads the
            // caller's states itself (it is also the only one that writes them), unless they are zero by contract.
            const bool cut = Tb > a.seg_tokens;
            // (with states that are zero by contract the first segment has nothing to read: the scan leaves its slot unwritten)
            if (kFull && (!a.zero_init || (cut && p > 0))) {
#pragma unroll
                for (int i = 0; i < NST; ++i) {
                    const float *src = cut ? a.ws_state + ((slot0 + static_cast<size_t>(p) * a.slot_mul * slot_step) * 2 + i) * D * D
                                           : (i ? a.S2 : a.S1) + sbh * D * D;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int j = 0; j < 16; ++j) acc[i][dt][j] = src[sbase + (32 * dt + 16 * (j >> 3) + (j & 7)) * D];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int j = 0; j < 16; ++j) acc[i][dt][j] = 0.f;
            }
            TIO *orow = static_cast<TIO *>(a.o) + seg0;
            const bool accum = kExt && a.accumulate;
            lds_barrier();   // operands of step 0 are ready
            if (kFull) rescale(acc, sm + O_ENT + static_cast<uint32_t>(8 * g) * 4, g, 32 * ct + ln);   // into the middle frame of step 0
            for (int n = 0; n < nsteps; n += 2) {
                if (kStage && n > 0) flush_rows(sm, 1, ct, lane, orow - sstep, rs, S, accum);
                consume(sm, 0, acc, ct, lane, orow, rs, valid_of(n), 0, accum);
                orow += sstep;
                lds_barrier();                    // step n consumed (two sets: and step n+1 ready)
                if (SETS == 1) lds_barrier();     // one set: step n+1 ready
                if (n + 1 < nsteps) {
                    if (kStage) flush_rows(sm, 0, ct, lane, orow - sstep, rs, S, accum);
                    consume(sm, SETS - 1, acc, ct, lane, orow, rs, valid_of(n + 1), 1, accum);
                    orow += sstep;
                }
                lds_barrier();
                if (SETS == 1) lds_barrier();
            }
            // the last step (every staged row has passed a barrier)
            if (kStage) flush_rows(sm, (nsteps - 1) & 1, ct, lane, orow - sstep, rs, valid_of(nsteps - 1), accum);
            // ---- write the states out ----
#pragma unroll
            for (int i = 0; i < NST; ++i) {
                float *dst = nullptr;
                if (kFull) {
                    if (t1 == Tb) dst = (i ? a.S2 : a.S1) + sbh * D * D;   // the segment with the last token
                } else {
                    // contribution of segment p goes to state slot p+1
                    dst = a.ws_state + ((slot0 + (p + 1) * slot_step) * 2 + i) * D * D;
                }
                if (dst) {
                    const uint32_t sb = opaque(static_cast<uint32_t>(8 * g) * D + 32 * ct + ln);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int j = 0; j < 16; ++j) dst[sb + (32 * dt + 16 * (j >> 3) + (j & 7)) * D] = acc[i][dt][j];
                }
            }
        } else {
            // =============================== producer ===============================
            const int pw = wave - CT;
            const float gm = a.gamma_per_head ? a.gamma_per_head[h] : a.gamma;
            float gsv[2] = {gm * a.scale, (1.0f - gm) * a.scale};
            if (kExt && a.explicit_w) {
                gsv[0] = (a.wa_per_head ? a.wa_per_head[h] : a.wa) * a.scale;
                gsv[1] = (a.wb_per_head ? a.wb_per_head[h] : a.wb) * a.scale;
            }
            const float lg[2] = {__builtin_amdgcn_logf(fabsf(gsv[0])), __builtin_amdgcn_logf(fabsf(gsv[1]))};
            const uint32_t sgn[2] = {gsv[0] < 0.f ? A::kSignBits : 0u, gsv[1] < 0.f ? A::kSignBits : 0u};
            if constexpr (kLineProd) {
                LineAddr pa(sm, pw, static_cast<uint32_t>(lane));
                pa.preact = a.gate_inv_tau != 0.f;
                pa.unit = pa.preact ? a.gate_inv_tau : kLog2e;
                const float lgs = pa.st ? lg[1] : lg[0];
                const uint32_t sgns = pa.st ? sgn[1] : sgn[0];
                float tot = 0.f;   // lane l: gate sum of column (state st, feature 64 fh + l) over the step whose operands come next
                const TIO *q0 = static_cast<const TIO *>(a.q) + seg0, *k0 = static_cast<const TIO *>(a.k) + seg0,
                          *v0 = static_cast<const TIO *>(a.v) + seg0;
                const TG *g0p = static_cast<const TG *>(pa.st ? a.g2 : a.g1) + seg0;
                const uint32_t lane_col = 64 * pa.fh + 8 * (lane & 7);
                // the lane offsets of a whole step never change; only a ragged last step clamps its rows
                uint32_t off_whole[TPT], offv_whole[2];
#pragma unroll
                for (int j = 0; j < TPT; ++j) off_whole[j] = (pa.sq * TPT + j) * rs + lane_col;
#pragma unroll
                for (int j = 0; j < 2; ++j) offv_whole[j] = (16 * pa.st + 2 * pa.sq + j) * rs + lane_col;
                auto src_of = [&](int n) -> LineSrc {   // step n, or the last step when n is past the end
                    const int m = n < nsteps ? n : nsteps - 1;
                    const size_t so = static_cast<size_t>(m) * sstep;
                    const uint32_t vm = static_cast<uint32_t>(valid_of(m));   // >= 1
                    LineSrc s;
                    s.q = q0 + so; s.k = k0 + so; s.v = v0 + so; s.g = g0p + so;
#pragma unroll
                    for (int j = 0; j < TPT; ++j) s.off[j] = off_whole[j];
#pragma unroll
                    for (int j = 0; j < 2; ++j) s.offv[j] = offv_whole[j];
                    if (vm < static_cast<uint32_t>(S)) {   // uniform
#pragma unroll
                        for (int j = 0; j < TPT; ++j) {
                            const uint32_t row = pa.sq * TPT + j;
                            s.off[j] = (row < vm ? row : vm - 1) * rs + lane_col;
                        }
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const uint32_t row = 16 * pa.st + 2 * pa.sq + j;
                            s.offv[j] = (row < vm ? row : vm - 1) * rs + lane_col;
                        }
                    }
                    return s;
                };
                auto load_gates_l = [&](LineGates &g, const LineSrc &s) {
#pragma unroll
                    for (int j = 0; j < TPT; ++j) g.g[j].load(s.g, s.off[j]);
                };
                LineIO r0, r1;
                LineGates g0, g1;
                LineScan s0, s1;
                load_gates_l(g0, src_of(0));
                load_gates_l(g1, src_of(1));
                {
                    const LineSrc s = src_of(0);
#pragma unroll
                    for (int j = 0; j < TPT; ++j) {
                        r0.k[j].load(s.k, s.off[j]);
                        r0.q[j].load(s.q, s.off[j]);
                    }
                    r0.v[0].load(s.v, s.offv[0]);
                    r0.v[1].load(s.v, s.offv[1]);
                }
                line_scan_a(pa, g0, valid_of(0), s0);
                {
                    float t[8];
                    line_scan_b_read(pa, t);
                    line_scan_b(pa, t, tot);
                    line_note_step(pa, tot, a.status);
                    // the caller's states enter the middle frame of step 0
                    lds_st<float>(sm + O_ENT + (pa.dec - (sm + O_DEC)), __builtin_amdgcn_exp2f(0.5f * pa.unit * tot));
                }
                line_scan_c(pa, s0);
                load_gates_l(g0, src_of(2));
                {
                    const LineSrc io = src_of(1), gs = src_of(3);
                    line_produce(pa, 0, r0, s0, valid_of(0), g1, s1, valid_of(1), lgs, sgns, tot, a.status, LineNext{r1, io, g1, gs});
                }
                lds_barrier();   // operands of step 0 are ready
                for (int n = 0; n < nsteps; n += 2) {
                    {
                        const LineSrc io = src_of(n + 2), gs = src_of(n + 4);
                        line_produce(pa, 1, r1, s1, valid_of(n + 1), g0, s0, valid_of(n + 2), lgs, sgns, tot, a.status,
                                     LineNext{r0, io, g0, gs});
                    }
                    lds_barrier();
                    {
                        const LineSrc io = src_of(n + 3), gs = src_of(n + 5);
                        line_produce(pa, 0, r0, s0, valid_of(n + 2), g1, s1, valid_of(n + 3), lgs, sgns, tot, a.status,
                                     LineNext{r1, io, g1, gs});
                    }
                    lds_barrier();
                }
                return;
            }
            float seg_decay = 0.f;   // lane l: log2 of the segment decay of (state l / 32, feature 32 pw + l % 32)
            float tot = 0.f;         // lane l: gate sum of that column over the step whose operands come next
            ProdAddr pa(sm, pw, static_cast<uint32_t>(lane));
            pa.preact = a.gate_inv_tau != 0.f;
            pa.unit = pa.preact ? a.gate_inv_tau : kLog2e;

            // k and v of an extended launch: Hkv heads, head h reads key/value head h / (H / Hkv)
            const uint32_t rskv = kExt ? static_cast<uint32_t>(a.Hkv) * D : rs;
            const size_t seg0kv = kExt ? (static_cast<size_t>(seq0 + t0) * a.Hkv + h / (a.H / a.Hkv)) * D : seg0;
            const size_t sstepkv = static_cast<size_t>(S) * rskv;
            const TIO *q0 = static_cast<const TIO *>(a.q) + seg0, *k0 = static_cast<const TIO *>(a.k) + seg0kv,
                      *v0 = static_cast<const TIO *>(a.v) + seg0kv;
            const TG *g10 = static_cast<const TG *>(a.g1) + seg0, *g20 = static_cast<const TG *>(a.g2) + seg0;
            const uint32_t lane_col = 32 * pw + 8 * (lane & 3);
            auto src_of = [&](int n) -> StepSrc {   // step n, or the last step when n is past the end
                const int m = n < nsteps ? n : nsteps - 1;
                const size_t so = static_cast<size_t>(m) * sstep;
                const int vm = valid_of(m);   // >= 1
                StepSrc s;
                const size_t sokv = static_cast<size_t>(m) * sstepkv;
                s.q = q0 + so; s.k = k0 + sokv; s.v = v0 + sokv; s.g1 = g10 + so; s.g2 = g20 + so;
#pragma unroll
                for (int j = 0; j < RPT; ++j) {
                    uint32_t row = pa.sg * RPT + j;
                    row = row < static_cast<uint32_t>(vm) ? row : static_cast<uint32_t>(vm - 1);
                    s.off[j] = row * rs + lane_col;
                    if (kExt) s.offkv[j] = row * rskv + lane_col;
                }
                return s;
            };

            // Software pipeline over the steps, two of everything (even / odd step): while the operands of step m are
            // prepared, q, k, v of step m + 1 stream in, the gates of step m + 1 are scanned and those of step m + 3
            // stream in.
            RawIO r0, r1;
            RawGates g0, g1;
            ScanOut s0, s1;
            load_gates(g0, src_of(0));
            load_gates(g1, src_of(1));
            load_io(r0, src_of(0));
            scan_a(pa, g0, valid_of(0), s0);
            {
                float t[SGN];
                scan_b_read(pa, t);
                scan_b(pa, t, tot);
                note_step(pa, tot, seg_decay, a.status);
                // the caller's states enter the middle frame of step 0
                lds_st<float>(sm + O_ENT + (pa.dec - (sm + O_DEC)), __builtin_amdgcn_exp2f(0.5f * pa.unit * tot));
            }
            scan_c(pa, s0);
            load_gates(g0, src_of(2));
            {
                const StepSrc io = src_of(1), gs = src_of(3);
                produce(pa, 0, r0, s0, valid_of(0), g1, s1, valid_of(1), lg, sgn, tot, seg_decay, a.status,
                        NextLoads{r1, io, g1, gs});
            }
            lds_barrier();   // operands of step 0 are ready
            for (int n = 0; n < nsteps; n += 2) {
                // consumers work on step n from set 0: prepare step n+1 into set 1
                if (SETS == 1) lds_barrier();     // one set: wait until step n is consumed
                {
                    const StepSrc io = src_of(n + 2), gs = src_of(n + 4);
                    produce(pa, SETS - 1, r1, s1, valid_of(n + 1), g0, s0, valid_of(n + 2), lg, sgn, tot, seg_decay,
                            a.status, NextLoads{r0, io, g0, gs});
                }
                lds_barrier();
                if (SETS == 1) lds_barrier();
                {
                    const StepSrc io = src_of(n + 3), gs = src_of(n + 5);
                    produce(pa, 0, r0, s0, valid_of(n + 2), g1, s1, valid_of(n + 3), lg, sgn, tot, seg_decay,
                            a.status, NextLoads{r1, io, g1, gs});
                }
                lds_barrier();
            }
            if (!kFull) {
                // log2 decay of segment p goes to decay slot p
                a.ws_decay[(slot0 + p * slot_step) * 2 * D + (lane >> 5) * D + 32 * pw + (lane & 31)] = seg_decay;
            }
        }
    }
};

// Wavefronts per SIMD the register budget is set for: two, except for the fp32 step loop at d = 64, whose one
// workgroup per compute unit (LDS) is one wavefront per SIMD and whose accumulators do not fit half the register file.
template <int D, class TIO, class TG, bool kFull, bool kExt, bool kBeta = false>
__global__ __launch_bounds__(4 * D, (D == 64 && sizeof(TIO) == 4 && kFull) ? 1 : 2) void prefill_kernel(PrefillArgs a)
{
    using K = Kern<D, TIO, TG, kFull, kExt, kBeta>;
    __shared__ __attribute__((aligned(16))) char smem[K::LDS_BYTES];
    K::run(a, lds_addr_of(smem));
}

// ---------------------------------------------------------------------------------------------
// Segment pre-pass of its own design for the common case: 16-bit io and gates, d = 128, two states.
//
// The state contribution of a segment of N tokens is U^i = sum_t diag(prod_{s > t} alpha^i_s) k_t^T v_t (Section 4.1,
// the state update unrolled to the end of the segment).  Walking the segment BACKWARDS, 32 tokens at a time, the
// exponent of every factor is a running suffix sum of log-gates: never positive, so nothing is centred and the
// accumulated state is never rescaled:
//     K~^i_t = k_t 2^{E^i_t},  E^i_t = sum_{s > t} log2 alpha^i_s  (<= 0)        U^i += (K~^i)^T V      per step.
// Inputs reach LDS as whole rows through loads that write LDS directly (no registers, 2 steps ahead of their use:
// 64 KB per workgroup in flight).  The suffix sums over the 32 tokens of a step are a product of a constant 0/1
// matrix with the tile of log-gates: the matrix unit evaluates them, exactly, and hands every lane one feature and 16
// tokens of it; a transposing LDS read delivers the keys in the same arrangement, and what is left for the vector unit
// is one fused multiply-add, one exponential, one multiply and half a pack per (token, feature, state): a third of
// what the producer wavefronts of the step-loop template spend on the same operands.
//
// All 8 wavefronts do both jobs: wavefront w prepares state w / 4, features 32 (w % 4) .. + 31, and multiplies
// state w / 4, columns 32 (w % 4) .. + 31 (64 accumulator registers).  One barrier per step: in interval n every
// wavefront prepares K~ of step n into one of two K~ buffers and then multiplies step n - 1, so the vector and the
// matrix work of neighbouring steps overlap across the wavefronts of a SIMD.
// LDS: 3 slots of (k, g1, g2) rows + 4 slots of v rows + 2 K~ buffers = 72 + 32 + 32 KB.  All rows as loaded, the
// 64-byte quarter q of row r at quarter position q ^ (r % 4) (every tensor is read transposed); K~ as in the
// step-loop template: [i D + feature][rho(token)], piece c of row R at c ^ ((R / 2) % 4).
// ---------------------------------------------------------------------------------------------
struct SegFast {
    static constexpr int D = 128, S = 32;
    static constexpr int NWAVE = 8, NT = 64 * NWAVE;
    static constexpr int LEAD = 2;                                     // steps between a load and its use
    static constexpr int KG_SLOTS = LEAD + 1, V_SLOTS = LEAD + 2;      // v lives one interval longer (it is multiplied one later)
    static constexpr uint32_t ROWB = D * 2, TEN = S * ROWB;            // a row, a tensor of one step (bytes)
    static constexpr uint32_t KG_BYTES = 3 * TEN;
    static constexpr uint32_t O_KG = 0, O_V = O_KG + KG_SLOTS * KG_BYTES, O_KT = O_V + V_SLOTS * TEN;
    static constexpr uint32_t KT_BYTES = 2 * D * S * 2;
    static constexpr uint32_t LDS_BYTES = O_KT + 2 * KT_BYTES;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// 16 bytes per lane from `base` (wavefront-uniform) + `voff` (per lane) into LDS at `lds` (uniform) + 16 * lane.
// The compiler does not know these loads: whoever reads the bytes waits with wait_loads<>() first.
// (M0 holds the LDS address; the compiler reserves that register for instructions of this kind and is told that it changes.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds16(uint32_t lds, uint32_t voff, const char *base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(base) : "m0", "memory");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier()   // at most N of this wavefront's loads still in flight; then the workgroup meets
{
    static_assert(N == 0 || N == 4, "one step of loads is 4 instructions per wavefront");
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ const char *uniform_ptr(const void *p)   // the same pointer, held in scalar registers
{
    const uint64_t x = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x)));
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x >> 32)));
    return reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
}
__global__ __launch_bounds__(SegFast::NT, 2) void segment_state_fast_kernel(PrefillArgs a)
{
    using F = SegFast;
    using A = ArithBf16;
    constexpr int D = F::D, S = F::S;
    __shared__ __attribute__((aligned(1024))) char smem[F::LDS_BYTES];
    const uint32_t sm = lds_addr_of(smem);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));

    // the work item: as Kern::run with kFull = false
    int bidx, h, p;
    size_t slot0, slot_step;
    if (a.list_full) {
        const int it = blockIdx.x / a.H;
        if (it >= a.seg_count[1]) return;
        const int2 e = a.list_pre[it];
        bidx = e.x;
        p = e.y;
        h = blockIdx.x % a.H;
        slot0 = static_cast<size_t>(a.seg_first[bidx]) * a.H + h;
        slot_step = a.H;
    } else {
        const int nseg = a.P - 1;
        const int bh = blockIdx.x / nseg;
        p = blockIdx.x % nseg;
        bidx = bh / a.H;
        h = bh % a.H;
        slot0 = bh;
        slot_step = gridDim.x / nseg;
    }
    const int sq = (a.cu && a.seq) ? a.seq[bidx] : bidx;
    const int64_t seq0 = a.cu ? static_cast<int64_t>(a.cu[sq]) : static_cast<int64_t>(bidx) * a.T;
    const int64_t Tb = a.cu ? static_cast<int64_t>(a.cu[sq + 1]) - seq0 : a.T;
    const int64_t t0 = static_cast<int64_t>(p) * a.seg_tokens;
    if (t0 + a.seg_tokens >= Tb) return;   // no segment follows: nobody needs this one's contribution (uniform exit)
    const int nsteps = static_cast<int>(a.seg_tokens / S);   // a segment with a successor is whole: a multiple of the chunk
    const uint32_t rs2 = static_cast<uint32_t>(a.H) * D * 2;   // bytes between consecutive tokens
    const size_t seg0 = (static_cast<size_t>(seq0 + t0) * a.H + h) * D * 2;
    const size_t step_bytes = static_cast<size_t>(S) * rs2;
    // k and v may have fewer heads (extended launches): head h reads key/value head h / (H / Hkv)
    const uint32_t rs2kv = static_cast<uint32_t>(a.Hkv) * D * 2;
    const size_t seg0kv = (static_cast<size_t>(seq0 + t0) * a.Hkv + h / (a.H / a.Hkv)) * D * 2;
    const size_t step_bytes_kv = static_cast<size_t>(S) * rs2kv;
    const char *pk = uniform_ptr(static_cast<const char *>(a.k) + seg0kv), *pv = uniform_ptr(static_cast<const char *>(a.v) + seg0kv),
               *pg1 = uniform_ptr(static_cast<const char *>(a.g1) + seg0), *pg2 = uniform_ptr(static_cast<const char *>(a.g2) + seg0);

    // ---- loading: wavefront w brings rows 4 w .. 4 w + 3 of every tensor of a step, lane l piece position l % 16 of row l / 16 ----
    const uint32_t drow = 4 * wave + (lane >> 4), dpos = lane & 15;
    const uint32_t dpiece = ((((dpos >> 2) ^ (drow & 3u)) << 2) | (dpos & 3u)) << 4;
    const uint32_t voff = drow * rs2 + dpiece, voff_kv = drow * rs2kv + dpiece;
    auto issue = [&](uint32_t kg_slot, uint32_t v_slot, int n) {   // step n of the walk = step nsteps - 1 - n of the segment
        const size_t off = static_cast<size_t>(nsteps - 1 - n) * step_bytes, off_kv = static_cast<size_t>(nsteps - 1 - n) * step_bytes_kv;
        const uint32_t kgb = sm + F::O_KG + kg_slot * F::KG_BYTES + wave * 1024;
        load_to_lds16(kgb, voff_kv, pk + off_kv);
        load_to_lds16(kgb + F::TEN, voff, pg1 + off);
        load_to_lds16(kgb + 2 * F::TEN, voff, pg2 + off);
        load_to_lds16(sm + F::O_V + v_slot * F::TEN + wave * 1024, voff_kv, pv + off_kv);
    };

    // Both jobs of wavefront w concern state st = w / 4 and the 32-tile ct = w % 4: features 32 ct .. of the keys and gates
    // when preparing, columns 32 ct .. of the values when multiplying.  A transposing read of staged rows hands lane
    // (ln, g) column 32 ct + ln and, for token block kb, the 8 tokens tau(kb, g, e) = 16 kb + 8 (e / 4) + 4 g + e % 4 --
    // an MFMA input fragment whose contraction index runs over the tokens in that order.
    const uint32_t st = wave >> 2, ct = wave & 3, ln = lane & 31, g = lane >> 5, l16 = lane & 15, vr = 4 * g + (l16 >> 2);
    const uint32_t tr_r = vr * F::ROWB + 64 * (ct ^ (vr & 3u)) + 32 * ((lane >> 4) & 1u) + 8 * (l16 & 3u);   // inside a staged tensor
    auto rows_frag = [&](uint32_t tensor, int kb) { return A::load_frag_tr(tensor + tr_r + 16 * kb * F::ROWB, 8 * F::ROWB); };
    // K~ rows: lane (ln, g) writes (preparing) and reads (multiplying) piece g + 2 kb of row st D + 32 tile + ln
    const uint32_t kt_r = sm + F::O_KT + (st * D + ln) * 64;
    const uint32_t kt_p[2] = {(g ^ ((ln >> 1) & 3u)) << 4, ((g + 2) ^ ((ln >> 1) & 3u)) << 4};

    // ---- preparing ----
    // The exponents of a step are suffix sums of its log-gates over the tokens: E[t][f] = sum_{t' > t} g[t'][f], a product
    // of a constant 0/1 matrix with the gate tile, which the matrix unit evaluates exactly (bf16 gates times 0 or 1, fp32
    // sums): tri[kb] is row ln of that matrix as the fragment whose contraction index runs over tau(kb, g, .).  The result
    // tile hands lane (ln, g) feature 32 ct + ln and, in register j, token 8 (j / 4) + 4 g + j % 4 = tau(j / 8, g, j % 8): the
    // order in which a transposing read delivers the keys, and 8 consecutive positions of a K~ row.
    A::Frag tri[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        u32x4 u;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t t_lo = 16 * kb + 8 * ((2 * w) >> 2) + 4 * g + ((2 * w) & 3), t_hi = t_lo + 1;
            u[w] = (t_lo > ln ? 0x3f80u : 0u) | (t_hi > ln ? 0x3f800000u : 0u);   // bf16 1.0 = 0x3f80
        }
        tri[kb].v = __builtin_bit_cast(bf16x8, u);
    }
    const bool preact = a.gate_inv_tau != 0.f;
    const float unit = preact ? a.gate_inv_tau : kLog2e;   // gate sums times this = log2 of a decay
    float carry = 0.f;   // gate sum over all later steps of the segment, feature 32 ct + ln of state st (the same in both lane groups)

    auto prepare = [&](uint32_t kg_slot, uint32_t kt_buf) {
        const uint32_t kbase = sm + F::O_KG + kg_slot * F::KG_BYTES, gbase = kbase + (1 + st) * F::TEN;
        A::Frag gf[2], kf[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) gf[kb] = rows_frag(gbase, kb);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kf[kb] = rows_frag(kbase, kb);
        f32x16 E;
#pragma unroll
        for (int j = 0; j < 16; ++j) E[j] = 0.f;
        float g_first;   // the gate of token tau(0, g, 0) = 4 g
        if (!preact) {
            A::mma(E, tri[0], gf[0]);
            A::mma(E, tri[1], gf[1]);
            g_first = __uint_as_float(__builtin_bit_cast(u32x4, gf[0].v)[0] << 16);
        } else {
            // pre-activations z -> tau log2 alpha (as Kern::activate); the result is not a bf16 number: it enters the
            // matrix unit as the sum of two (hi + lo: 16 mantissa bits)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const u32x4 zw = __builtin_bit_cast(u32x4, gf[kb].v);
                u32x4 hi, lo;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    float x[2] = {__uint_as_float(zw[w] << 16), __uint_as_float(zw[w] & 0xffff0000u)};
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float y = x[e] * kLog2e;
                        x[e] = fminf(y, 0.f) - __builtin_amdgcn_logf(1.0f + __builtin_amdgcn_exp2f(-__builtin_fabsf(y)));
                    }
                    if (kb == 0 && w == 0) g_first = x[0];
                    hi[w] = A::pack2(x[0], x[1]);
                    lo[w] = A::pack2(x[0] - __uint_as_float(hi[w] << 16), x[1] - __uint_as_float(hi[w] & 0xffff0000u));
                }
                A::Frag fh, fl;
                fh.v = __builtin_bit_cast(bf16x8, hi);
                fl.v = __builtin_bit_cast(bf16x8, lo);
                A::mma(E, tri[kb], fh);
                A::mma(E, tri[kb], fl);
            }
        }
        // gate sum of the whole step = E[token 0] + g[token 0]: lane group 0 has it, group 1 fetches it
        const float tot = __int_as_float(__builtin_amdgcn_ds_bpermute(static_cast<int>(ln << 2), __float_as_int(E[0] + g_first)));
        const float cu = carry * unit;
        carry += tot;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const u32x4 kw = __builtin_bit_cast(u32x4, kf[kb].v);
            u32x4 out;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float k0 = __uint_as_float(kw[w] << 16), k1 = __uint_as_float(kw[w] & 0xffff0000u);
                out[w] = A::pack2(k0 * __builtin_amdgcn_exp2f(fmaf(E[8 * kb + 2 * w], unit, cu)),
                                  k1 * __builtin_amdgcn_exp2f(fmaf(E[8 * kb + 2 * w + 1], unit, cu)));
            }
            lds_st<u32x4>(kt_r + kt_buf * F::KT_BYTES + 32 * ct * 64 + kt_p[kb], out);
        }
    };

    // ---- multiplying: U[st][:, 32 ct ..] += K~^T V ----
    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[dt][j] = 0.f;
    auto multiply = [&](uint32_t v_slot, uint32_t kt_buf) {
        A::Frag vf[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) vf[kb] = rows_frag(sm + F::O_V + v_slot * F::TEN, kb);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                A::mma(acc[dt], A::load_frag(kt_r + kt_buf * F::KT_BYTES + 32 * dt * 64 + kt_p[kb]), vf[kb]);
    };

    // ---- the walk: interval n prepares step n and multiplies step n - 1 ----
    issue(0, 0, 0);
    if (nsteps > 1) issue(1, 1, 1);
    uint32_t kg_n = 0, v_n = 0;          // slots of step n
    uint32_t kg_i = 2, v_i = 2;          // slots of step n + LEAD
    for (int n = 0; n <= nsteps; ++n) {
        // step n has landed (the loads of step n + 1 may still be in flight); K~ of step n - 1 is complete; the slots
        // and the K~ buffer that this interval overwrites have been read by everyone
        if (n + 1 < nsteps) wait_loads_and_barrier<4>();
        else wait_loads_and_barrier<0>();
        if (n + F::LEAD < nsteps) issue(kg_i, v_i, n + F::LEAD);
        if (n < nsteps) prepare(kg_n, static_cast<uint32_t>(n) & 1u);
        if (n >= 1) multiply(v_n == 0 ? F::V_SLOTS - 1 : v_n - 1, static_cast<uint32_t>(n - 1) & 1u);
        kg_n = kg_n + 1 == F::KG_SLOTS ? 0 : kg_n + 1;
        v_n = v_n + 1 == F::V_SLOTS ? 0 : v_n + 1;
        kg_i = kg_i + 1 == F::KG_SLOTS ? 0 : kg_i + 1;
        v_i = v_i + 1 == F::V_SLOTS ? 0 : v_i + 1;
    }

    // ---- contribution of segment p -> state slot p + 1; its log2 decay -> decay slot p ----
    {
        float *dst = a.ws_state + ((slot0 + (p + 1) * slot_step) * 2 + st) * D * D + (4 * g) * D + 32 * ct + ln;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int j = 0; j < 16; ++j) dst[(32 * dt + 8 * (j >> 2) + (j & 3)) * D] = acc[dt][j];
        if (g == 0) a.ws_decay[(slot0 + p * slot_step) * 2 * D + st * D + 32 * ct + ln] = carry * unit;
    }
}

// Work lists for packed sequences (one workgroup): sequence b has ceil(T_b / seg_tokens) segments;
// seg_first = exclusive prefix sum of that over the sequences, list_full = every (sequence, segment),
// list_pre = those with a successor.  Thread t takes a contiguous run of sequences.
__global__ __launch_bounds__(256) void segment_list_kernel(const int32_t *__restrict__ cu, const int32_t *__restrict__ seq,
                                                           int B, int64_t seg_tokens,
                                                           int32_t *__restrict__ seg_first,
                                                           int32_t *__restrict__ seg_count, int2 *__restrict__ list_full,
                                                           int2 *__restrict__ list_pre, int cap_full, int cap_pre)
{
    __shared__ int s_sum[256];
    const int t = threadIdx.x;
    const int per = (B + 255) / 256;
    const int b0 = t * per, b1 = (b0 + per < B) ? b0 + per : B;
    auto segments_of = [&](int b) -> int {
        const int sq = seq ? seq[b] : b;
        const int64_t Tb = static_cast<int64_t>(cu[sq + 1]) - cu[sq];
        return Tb > 0 ? static_cast<int>((Tb + seg_tokens - 1) / seg_tokens) : 0;
    };
    int mine = 0, mine_seq = 0;   // segments, and sequences with at least one, in this thread's run
    for (int b = b0; b < b1; ++b) {
        const int n = segments_of(b);
        mine += n;
        mine_seq += n > 0;
    }
    // exclusive scans over the 256 threads of (segments) and (segments - non-empty sequences) = entries of list_pre
    s_sum[t] = mine;
    __syncthreads();
    int before = 0, before_seq = 0;
    for (int u = 0; u < t; ++u) before += s_sum[u];
    __syncthreads();
    s_sum[t] = mine_seq;
    __syncthreads();
    for (int u = 0; u < t; ++u) before_seq += s_sum[u];
    int at = before, at_pre = before - before_seq;
    for (int b = b0; b < b1; ++b) {
        const int n = segments_of(b);
        seg_first[b] = at;
        // the capacities hold whenever the offsets add up to the total the caller gave; offsets that do not
        // must not write past the lists (the segments that do not fit are dropped)
        for (int p = 0; p < n; ++p) {
            if (at + p < cap_full) list_full[at + p] = make_int2(b, p);
            if (p + 1 < n) {
                if (at_pre < cap_pre) list_pre[at_pre] = make_int2(b, p);
                ++at_pre;
            }
        }
        at += n;
    }
    if (t == 255) {
        seg_first[B] = at;
        seg_count[0] = at < cap_full ? at : cap_full;
        seg_count[1] = at_pre < cap_pre ? at_pre : cap_pre;
    }
}

// Elementwise scan over the segments of every (sequence, head) that has more than one: s_0 = caller's state goes to
// the slot of segment 0; s_{p+1} = 2^{decay_p} s_p + U_p goes to the slot of segment p+1, where the segment_state
// kernel had left U_p.  The chunk loop then takes every initial state of such a sequence from the slots.
template <int D>
__global__ __launch_bounds__(256) void segment_scan_kernel(const float *__restrict__ S1, const float *__restrict__ S2,
                                                           float *__restrict__ ws_state,
                                                           const float *__restrict__ ws_decay, int BH, int P,
                                                           const int32_t *__restrict__ cu,
                                                           const int32_t *__restrict__ seq,
                                                           const int32_t *__restrict__ slot,
                                                           const int32_t *__restrict__ seg_first, int H,
                                                           int64_t seg_tokens, int zero_init, int beta)
{
    // one thread per 4 adjacent columns of one (bh, state, row)
    const size_t n4 = static_cast<size_t>(BH) * 2 * D * (D / 4);
    const size_t idx = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n4) return;
    const int c4 = static_cast<int>(idx % (D / 4));
    const size_t r = idx / (D / 4);  // (bh*2 + i)*D + row
    const int row = static_cast<int>(r % D);
    const size_t bi = r / D;         // bh*2 + i
    const int i = static_cast<int>(bi & 1);
    if (beta && i) return;   // beta mode: one state; the second slot of decays holds the log2 decays of its columns
    const size_t bh = bi >> 1;
    const size_t b = bh / H, h = bh % H;
    size_t slot0 = bh, slot_step = BH;
    if (cu) {   // a shorter sequence has fewer segments, an empty one none
        const size_t sq = seq ? static_cast<size_t>(seq[b]) : b;
        const int64_t Tb = static_cast<int64_t>(cu[sq + 1]) - cu[sq];
        const int64_t Pb = Tb > 0 ? (Tb + seg_tokens - 1) / seg_tokens : 0;
        if (Pb < P) P = static_cast<int>(Pb);
        if (P <= 1) return;
        slot0 = static_cast<size_t>(seg_first[b]) * H + h;
        slot_step = H;
    }
    const size_t sbh = static_cast<size_t>(slot ? slot[b] : b) * H + h;
    const float *src = (i ? S2 : S1) + (sbh * D + row) * D + c4 * 4;
    float4 s = zero_init ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4 *>(src);
    const size_t in_slot = (static_cast<size_t>(i) * D + row) * D + c4 * 4;   // this thread's place inside a slot
    if (P <= 1) return;
    if (!zero_init) *reinterpret_cast<float4 *>(ws_state + slot0 * 2 * D * D + in_slot) = s;   // zero states: segment 0 starts from registers set to zero
    for (int p = 0; p + 1 < P; ++p) {
        const float *dslot = ws_decay + (slot0 + p * slot_step) * 2 * D;
        const float dr = dslot[i * D + row];
        float4 dec = make_float4(dr, dr, dr, dr);
        if (beta) {
            const float4 dc = *reinterpret_cast<const float4 *>(dslot + D + c4 * 4);
            dec.x += dc.x; dec.y += dc.y; dec.z += dc.z; dec.w += dc.w;
        }
        dec.x = __builtin_amdgcn_exp2f(dec.x); dec.y = __builtin_amdgcn_exp2f(dec.y);
        dec.z = __builtin_amdgcn_exp2f(dec.z); dec.w = __builtin_amdgcn_exp2f(dec.w);
        float4 *u = reinterpret_cast<float4 *>(ws_state + (slot0 + (p + 1) * slot_step) * 2 * D * D + in_slot);
        const float4 x = *u;
        s.x = fmaf(dec.x, s.x, x.x);
        s.y = fmaf(dec.y, s.y, x.y);
        s.z = fmaf(dec.z, s.z, x.z);
        s.w = fmaf(dec.w, s.w, x.w);
        if (!(zero_init && p == 0)) *u = s;   // from zero states the first slot already holds its result
    }
}


template <int D, class TIO, class TG, bool kExt, bool kBeta = false>
hipError_t launch_x(const dsla_desc &d, const PrefillPlan &plan, PrefillArgs &a, hipStream_t stream)
{
    const int BH = d.B * d.H;
    // The pre-pass and the scan see every segment but the last as R pieces (R = plan.pre_split; 1 with work lists):
    // to them the sequence has R (P - 1) + 1 segments of segment_tokens / R tokens, the last one longer, which neither
    // of them touches.  The chunk loop then finds the state entering its segment p in slot R p.
    const int R = plan.segments > 1 ? plan.pre_split : 1;
    PrefillArgs af = a;
    af.P = R * (plan.segments - 1) + 1;
    af.seg_tokens = a.seg_tokens / R;
    a.slot_mul = R;
    // workgroups of the two big kernels: one per (segment, sequence, head); with work lists one per (list entry, head)
    const unsigned grid_pre = a.list_full ? static_cast<unsigned>(plan.max_pre_items * d.H)
                                          : static_cast<unsigned>(BH * (af.P - 1));
    const unsigned grid_full = a.list_full ? static_cast<unsigned>(plan.max_items * d.H)
                                           : static_cast<unsigned>(BH * plan.segments);
    hipError_t err = hipSuccess;
    if (plan.segments > 1) {
        if (a.list_full) {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_LIST, stream);
            DSLA_LAUNCH(ps, segment_list_kernel, dim3(1), dim3(256), 0, stream, a.cu, a.seq, d.B, a.seg_tokens,
                               const_cast<int32_t *>(a.seg_first), const_cast<int32_t *>(a.seg_count),
                               const_cast<int2 *>(a.list_full), const_cast<int2 *>(a.list_pre),
                               static_cast<int>(plan.max_items), static_cast<int>(plan.max_pre_items));
            err = hipGetLastError();
            if (err != hipSuccess) return err;
        }
        if (grid_pre > 0) {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_STATE, stream);
            // the pre-pass of its own design where it is built; its per-lane offsets inside a step are 32-bit
            constexpr bool kFast = D == SegFast::D && std::is_same<TIO, bf16_t>::value && std::is_same<TG, bf16_t>::value && !kBeta;
            if (kFast && static_cast<int64_t>(d.H) * D * 2 * SegFast::S < (int64_t{1} << 31))
                DSLA_LAUNCH(ps, segment_state_fast_kernel, dim3(grid_pre), dim3(SegFast::NT), 0, stream, af);
            else
                DSLA_LAUNCH(ps, (prefill_kernel<D, TIO, TG, false, kExt, kBeta>), dim3(grid_pre), dim3(4 * D), 0, stream, af);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
        {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_SCAN, stream);
            const size_t n4 = static_cast<size_t>(BH) * 2 * D * (D / 4);
            DSLA_LAUNCH(ps, (segment_scan_kernel<D>), dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0,
                               stream, a.S1, a.S2, a.ws_state, a.ws_decay, BH, af.P, a.cu, a.seq, a.slot,
                               a.seg_first, a.H, af.seg_tokens, a.zero_init, kBeta ? 1 : 0);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
    }
    {
        ProfileScope ps(DSLA_KERNEL_PREFILL_CHUNK_LOOP, stream);
        DSLA_LAUNCH(ps, (prefill_kernel<D, TIO, TG, true, kExt, kBeta>), dim3(grid_full), dim3(4 * D), 0, stream, a);
    }
    err = hipGetLastError();
    return err;
}

// Ordinary launches keep the lean kernels; explicit blend coefficients, grouped key/value heads and accumulation
// into o select the extended ones.
template <int D, class TIO, class TG>
hipError_t launch_t(const dsla_desc &d, const PrefillPlan &plan, PrefillArgs &a, hipStream_t stream)
{
    if (a.beta) return launch_x<D, TIO, TG, true, true>(d, plan, a, stream);
    if (a.explicit_w || a.accumulate || a.Hkv != a.H) return launch_x<D, TIO, TG, true>(d, plan, a, stream);
    return launch_x<D, TIO, TG, false>(d, plan, a, stream);
}

template <int D, class TIO>
hipError_t launch_g(const dsla_desc &d, const PrefillPlan &plan, PrefillArgs &a, hipStream_t stream)
{
    if (d.gate_dtype == DSLA_BF16) return launch_t<D, TIO, bf16_t>(d, plan, a, stream);
    return launch_t<D, TIO, float>(d, plan, a, stream);
}

// The chunk length only sets the granularity of the segment split; the kernels step through 32 tokens at a time.
bool combo_built(int D, int C, int io)
{
    return (io == DSLA_BF16 || io == DSLA_F32) && (D == 64 || D == 128) && (C == 32 || C == 64 || C == 128);
}

}  // namespace

namespace {
// Fills the plan from the chunk length, the number of segments P the longest sequence is cut into, and its length.
void finish_plan(const dsla_desc &d, int C, int64_t P, int64_t nchunks, bool may_split, PrefillPlan *plan)
{
    const int D = d.d_k;
    const int64_t BH = static_cast<int64_t>(d.B) * d.H;
    if (P < 1) P = 1;
    if (P > nchunks) P = nchunks;
    const int64_t cps = (nchunks + P - 1) / P;
    P = (nchunks + cps - 1) / cps;
    plan->chunk = C;
    plan->segments = static_cast<int>(P);
    plan->segment_tokens = cps * C;
    plan->state_elems = static_cast<size_t>(BH) * D * D;
    plan->max_items = plan->max_pre_items = 0;
    plan->ws_lists_bytes = 0;
    // The pre-pass has one workgroup per (segment but the last, sequence, head).  With two segments that is at most
    // half of the compute units (65 .. 128 heads in all; short sequences): it then works on the two halves of the first
    // segment and the scan combines them: measured at B H = 128, T = 16384 the pre-pass streams at 3.7 TB/s from 128
    // workgroups and at 5.7 TB/s from 256.  With more segments the longer scan costs what the shorter pieces gain
    // (B H = 32, T = 1024, four segments: pre-pass - 2 us, scan + 5 us).  A caller who names the number of segments
    // gets exactly those.
    plan->pre_split = (may_split && P == 2 && cps % 2 == 0 && cps * C >= 256 && BH * 2 <= ((D == 64) ? 512 : 256)) ? 2 : 1;
    if (P > 1) {
        const int64_t pieces = plan->pre_split * (P - 1) + 1;
        plan->ws_state_bytes = static_cast<size_t>(pieces) * plan->state_elems * 2 * sizeof(float);
        plan->ws_decay_bytes = ((static_cast<size_t>(pieces - 1) * BH * 2 * D * sizeof(float)) + 255) / 256 * 256;
    } else {
        plan->ws_state_bytes = 0;
        plan->ws_decay_bytes = 0;
    }
    plan->ws_total_bytes = plan->ws_state_bytes + plan->ws_decay_bytes;
}
int plan_chunk(const dsla_desc &d)
{
    if (d.d_k != d.d_v) return 0;
    int C = d.chunk;
    if (C == 0) C = combo_built(d.d_k, 64, d.io_dtype) ? 64 : 32;
    return combo_built(d.d_k, C, d.io_dtype) ? C : 0;
}
}  // namespace

bool prefill_plan(const dsla_desc &d, int64_t T, PrefillPlan *plan)
{
    const int C = plan_chunk(d);
    if (!C) return false;
    const int64_t nchunks = (T + C - 1) / C;
    const int64_t BH = static_cast<int64_t>(d.B) * d.H;
    int64_t P;
    if (d.segments > 0) {
        P = d.segments;
    } else {
        // enough workgroups to cover the 256 compute units (two per unit for the small head size),
        // but at least 4 chunks per segment so that the extra segment_state pass stays cheap
        const int64_t target = (d.d_k == 64) ? 512 : 256;
        P = target / BH;
        if (P > nchunks / 4) P = nchunks / 4;
    }
    finish_plan(d, C, P, nchunks, d.segments <= 0, plan);
    return true;
}

// Packed sequences of different lengths share one segment length; a sequence of length T_b has
// ceil(T_b / segment_tokens) segments.  The segment length is chosen so that all sequences together make about
// one workgroup per compute unit, the same rule as above on the total instead of a common length (measured on
// mixed batches: twice as many segments gain on some mixes and lose on others, within 10 %).
// The kernels find their work in lists built on the device (the lengths are not known here); list and workspace
// sizes are worst cases: sum_b ceil(T_b / L) <= total_T / L + B segments, of which at most total_T / L have a
// successor.
bool prefill_plan_varlen(const dsla_desc &d, int64_t total_T, int64_t max_T, PrefillPlan *plan)
{
    const int C = plan_chunk(d);
    if (!C) return false;
    const int64_t nchunks = (max_T + C - 1) / C;
    int64_t P;
    if (d.segments > 0) {
        P = d.segments;
    } else {
        const int64_t target = (d.d_k == 64) ? 512 : 256;
        int64_t cps = (total_T * d.H / target + C - 1) / C;   // chunks per segment
        if (cps < 4) cps = 4;
        P = (nchunks + cps - 1) / cps;
    }
    finish_plan(d, C, P, nchunks, false, plan);
    if (plan->segments > 1) {
        const int D = d.d_k;
        auto up = [](size_t n) { return (n + 255) / 256 * 256; };
        plan->max_pre_items = total_T / plan->segment_tokens;
        plan->max_items = plan->max_pre_items + d.B;
        const size_t slots = static_cast<size_t>(plan->max_items) * d.H;
        plan->ws_state_bytes = slots * 2 * D * D * sizeof(float);
        plan->ws_decay_bytes = up(slots * 2 * D * sizeof(float));
        plan->ws_lists_bytes = up((static_cast<size_t>(d.B) + 1) * 4) + 256 + up(plan->max_items * 8) +
                               up(plan->max_pre_items * 8);
        plan->ws_total_bytes = plan->ws_state_bytes + plan->ws_decay_bytes + plan->ws_lists_bytes;
    }
    return true;
}

hipError_t launch_prefill(const dsla_desc &d, const PrefillPlan &plan, int64_t T, const int32_t *cu_seqlens,
                          const int32_t *seq_index, const int32_t *state_slot, const void *q, const void *k, const void *v, const void *g1,
                          const void *g2, float *S1, float *S2, void *o, void *workspace, hipStream_t stream,
                          const PrefillExt *ext)
{
    PrefillArgs a;
    a.slot_mul = 1;
    a.Hkv = ext ? ext->Hkv : d.H;
    a.explicit_w = ext ? 1 : 0;
    a.accumulate = ext ? ext->accumulate : 0;
    a.beta = ext ? ext->beta : 0;
    a.wa = ext ? ext->wa : 0.f;
    a.wb = ext ? ext->wb : 0.f;
    a.wa_per_head = ext ? ext->wa_per_head : nullptr;
    a.wb_per_head = ext ? ext->wb_per_head : nullptr;
    a.q = q; a.k = k; a.v = v; a.g1 = g1; a.g2 = g2; a.o = o;
    a.S1 = S1; a.S2 = S2;
    a.ws_state = static_cast<float *>(workspace);
    a.ws_decay = plan.segments > 1
                     ? reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.ws_state_bytes)
                     : nullptr;
    a.gamma_per_head = d.gamma_per_head;
    a.cu = cu_seqlens;
    a.seq = seq_index;
    a.slot = state_slot;
    a.seg_first = a.seg_count = nullptr;
    a.list_full = a.list_pre = nullptr;
    if (plan.max_items > 0) {   // packed sequences, more than one segment: carve the work lists
        auto up = [](size_t n) { return (n + 255) / 256 * 256; };
        char *w = static_cast<char *>(workspace) + plan.ws_state_bytes + plan.ws_decay_bytes;
        a.seg_first = reinterpret_cast<int32_t *>(w);
        w += up((static_cast<size_t>(d.B) + 1) * 4);
        a.seg_count = reinterpret_cast<int32_t *>(w);
        w += 256;
        a.list_full = reinterpret_cast<int2 *>(w);
        w += up(plan.max_items * 8);
        a.list_pre = reinterpret_cast<int2 *>(w);
    }
    a.T = T;
    a.seg_tokens = plan.segment_tokens;
    a.H = d.H;
    a.P = plan.segments;
    a.zero_init = d.zero_init != 0;
    a.status = d.status;
    a.gamma = d.gamma;
    a.scale = d.scale;
    a.gate_inv_tau = d.gate_mode == DSLA_GATE_PREACT ? 1.0f / d.tau : 0.f;
    const int D = d.d_k;
    if (d.io_dtype == DSLA_BF16) {
        if (D == 128) return launch_g<128, bf16_t>(d, plan, a, stream);
        if (D == 64) return launch_g<64, bf16_t>(d, plan, a, stream);
    } else {
        if (D == 128) return launch_g<128, float>(d, plan, a, stream);
        if (D == 64) return launch_g<64, float>(d, plan, a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace dsla
