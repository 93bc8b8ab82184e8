// Chunked DSLA prefill for gfx950 (paper Section 4.1: state-update equation and blended
// read-out, evaluated C tokens at a time).
//
// Chunk algebra (local positions r, s = 1..C inside a chunk, b^i_r = sum_{tau<=r} log2 alpha^i_tau,
// S^i = state entering the chunk, gamma_1 = gamma, gamma_2 = 1 - gamma):
//   o_r   = sum_i gamma_i scale (q_r * 2^{b^i_r}) S^i                       (read-out of carried state)
//         + sum_{s<=r} [ sum_i gamma_i scale (q_r * 2^{b^i_r}) . (k_s * 2^{-b^i_s}) ] v_s   (inside the chunk)
//   S^i  <- diag(2^{b^i_C}) S^i + sum_s (k_s * 2^{b^i_C - b^i_s})^T v_s
// which is the token recurrence regrouped; every bracket is a dense contraction and runs on MFMA.
// With Qc = [gamma_1 q~^1 | gamma_2 q~^2] and Kc = [k~^1 | k~^2] (width 2 d_k) the blend of the two
// states is part of the contraction: scores = Qc Kc^T, carried read-out = Qc [S^1; S^2].
//
// Parallel decomposition.  A sequence is cut into P segments so that B*H*P workgroups fill the
// chip.  (1) segment_state: every segment but the last computes, from a zero state, its state
// contribution U and its total log-decay.  (2) segment_scan: an elementwise scan over segments
// turns these into the true state entering each segment.  (3) chunk_loop: every segment runs the
// fused chunk loop from its true initial state and writes o; the last segment writes the final
// states.  P = 1 runs (3) alone.
//
// Workgroup = D/32 wavefronts (D = d_k = d_v).  Wavefront w owns state columns [32w, 32w+32) of
// both states for all d_k rows, as fp32 MFMA accumulators (tiles with m = state row, n = column).
// Because an MFMA accumulator tile and an MFMA input fragment both index lanes by the tile column,
// those accumulators are fed back as the input fragment of the carried read-out without passing
// through LDS; the partner operand is stored in LDS with the matching order of the contraction
// index (bits 2 and 3 of the feature index swapped).
#include <cstdio>
#include <type_traits>

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

// Development aid, compiled out unless DSLA_PHASE_CLOCKS is defined: one lane of workgroup 0 adds up the
// shader clock spent between phase marks and the launcher prints the totals.
#ifdef DSLA_PHASE_CLOCKS
struct PhaseClock {
    long long acc[12];
    long long last;
    __device__ __forceinline__ void start()
    {
        for (int n = 0; n < 12; ++n) acc[n] = 0;
        last = __builtin_amdgcn_s_memtime();
    }
    __device__ __forceinline__ void mark(int n)
    {
        const long long now = __builtin_amdgcn_s_memtime();
        acc[n] += now - last;
        last = now;
    }
    __device__ __forceinline__ void flush(long long *dbg) const
    {
        if (blockIdx.x == 0 && (threadIdx.x & 63) == 0 && dbg)
            for (int n = 0; n < 12; ++n) dbg[(threadIdx.x >> 6) * 12 + n] = acc[n];
    }
};
#else
struct PhaseClock {
    __device__ __forceinline__ void start() {}
    __device__ __forceinline__ void mark(int) {}
};
#endif

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

// staged output row (8 elements in LDS) -> global, uniform base + 32-bit lane offset
__device__ __forceinline__ void store8_global(bf16_t *base, uint32_t elem_off, uint32_t lds8)
{
    *reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(base) + elem_off * 2u) = lds_ld<u32x4>(lds8);
}
__device__ __forceinline__ void store8_global(float *base, uint32_t elem_off, uint32_t lds8)
{
    char *p = reinterpret_cast<char *>(base) + elem_off * 4u;
    *reinterpret_cast<f32x4 *>(p) = lds_ld<f32x4>(lds8);
    *reinterpret_cast<f32x4 *>(p + 16) = lds_ld<f32x4>(lds8 + 16);
}

// Software-pipelined sequence of N steps: the LDS fragment of step s + DEPTH is requested before the
// MFMA of step s is issued, so that LDS latency overlaps DEPTH matrix instructions.  Fully unrolled.
template <int N, int DEPTH, class ARITH, class AddrF, class StepF>
__device__ __forceinline__ void pipelined_steps(AddrF addr, StepF step)
{
    typename ARITH::Frag buf[DEPTH];
#pragma unroll
    for (int i = 0; i < DEPTH && i < N; ++i) buf[i] = ARITH::load_frag(addr(i));
#pragma unroll
    for (int s = 0; s < N; ++s) {
        const typename ARITH::Frag cur = buf[s % DEPTH];
        if (s + DEPTH < N) buf[s % DEPTH] = ARITH::load_frag(addr(s + DEPTH));
        step(s, cur);
    }
}

// ---------------------------------------------------------------------------------------------
struct PrefillArgs {
    const void *q, *k, *v, *g1, *g2;
    void *o;
    float *S1, *S2;          // caller's states
    float *ws_state;         // [P][BH][2][D][D] fp32 (P > 1)
    float *ws_decay;         // [P-1][BH][2][D] fp32, log2 of the segment decay (P > 1)
    const float *gamma_per_head;
    int64_t T;
    int64_t seg_tokens;
    int H;
    int P;
    float gamma, scale;
#ifdef DSLA_PHASE_CLOCKS
    long long *dbg;
#endif
};

// Workgroup layout.  A group of 2 D threads (D/32 wavefronts) prepares the operands of one state and owns
// that state in the contractions; inside a group, wavefront ct owns state columns [32 ct, 32 ct + 32).
// The chunk loop (kFull) runs both states in one workgroup of two groups, because the read-out blends
// them.  The segment pre-pass (!kFull) needs no blend: one state per workgroup of one group, so that
// several small workgroups share a compute unit and overlap each other's phases.
template <int D, int C, class TIO, class TG, bool kFull>
struct Kern {
    using A = ArithOf<TIO>;
    using Frag = typename A::Frag;
    using Row8 = typename A::Row8;
    static constexpr int ESZ = A::ESZ;

    static constexpr int CT = D / 32;       // column tiles = wavefronts per group
    static constexpr int GROUPS = kFull ? 2 : 1;   // wavefront groups = states handled by one workgroup
    static constexpr int NW = GROUPS * CT;  // wavefronts
    static constexpr int NT = 64 * NW;      // threads (4 D with both states, 2 D with one)
    static constexpr int GT = 2 * D;        // threads per group
    static constexpr int VW = kFull ? 4 : 8;   // v columns per thread (a group covers D/2 or all D columns)
    static constexpr int DG = D / 8;        // feature groups of 8
    static constexpr int SG = GT / DG;      // token groups (16)
    static constexpr int RPT = C / SG;      // tokens per thread
    static constexpr int QP = 2 * D + 8;    // pitch of row-layout operands (elements)
    static constexpr int TP = C + 8;        // pitch of token-contiguous operands (elements)
    static constexpr int OP = D + 8;        // pitch of the output staging tile
    static constexpr int NC16 = C / 8;      // 8-element column groups in a token-contiguous row
    static constexpr int RT = C / 32;       // 32-token tiles in a chunk
    static constexpr int KB = C / 16;       // contraction blocks over tokens
    static constexpr int DT = D / 32;       // 32-row tiles of a state
    static constexpr int NTILE = RT * (RT + 1) / 2;  // score tiles on or below the diagonal
    static constexpr int XS = (RT == 2) ? NW : CT;   // exchange slots: all wavefronts send (RT = 2) or group 1 only
    static_assert(SG == 16 && (RPT == 2 || RPT == 4), "chunk must be 32 or 64");
    static_assert(!kFull || NTILE <= NW, "one score tile per wavefront");

    // LDS map (byte offsets from the start of the block's LDS allocation)
    static constexpr uint32_t QS = 0;                                             // [token][i*D + d]  gamma_i scale q 2^{b}
    static constexpr uint32_t KS = QS + (kFull ? C * QP * ESZ : 0);               // [token][i*D + d]  k 2^{-b}
    static constexpr uint32_t KT = KS + (kFull ? C * QP * ESZ : 0);               // [i*D + rho(d)][token]  k 2^{bC-b}
    static constexpr uint32_t VT = KT + GROUPS * D * TP * ESZ;                    // [column][token]  v
    static constexpr uint32_t AS = VT + D * TP * ESZ;                             // [query][key] blended masked scores
    static constexpr uint32_t CS = AS + (kFull ? C * TP * ESZ : 0);               // float [i][token group][d] gate scan
    static constexpr uint32_t BC = CS + GROUPS * SG * D * 4;                      // float [GROUPS D] log2 chunk decay
    static constexpr uint32_t DEC = BC + GROUPS * D * 4;                          // float [GROUPS D] 2^{bC}
    static constexpr uint32_t LDS_BYTES = DEC + GROUPS * D * 4;
    static constexpr uint32_t XB = KS;   // partial-output exchange (float4 [XS][4][64]) reuses Ks after the scores
    static constexpr uint32_t OS = QS;   // output staging tile [token][OP] reuses Qs after the read-out
    static_assert(!kFull || XS * 4096 <= C * QP * ESZ, "exchange buffer fits in Ks");
    static_assert(!kFull || C * OP <= C * QP, "staging tile fits in Qs");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 compute unit");

    // swizzled offset inside a token-contiguous row: 8-element column group XOR (row / 8)
    static __device__ __forceinline__ uint32_t tcol(uint32_t row, uint32_t s)
    {
        return ((((s >> 3) ^ (row >> 3)) & (NC16 - 1)) << 3) | (s & 7);
    }
    // Kt row order: feature d sits in row rho(d) (bits 2 and 3 of d swapped).  With this order, accumulator
    // register j of lane group g in a 32-row state tile holds feature 16*(j/8) + 8*g + (j%8) of the tile:
    // the 8 registers of one half of the tile are 8 consecutive features, exactly one MFMA input fragment.

    // Inputs of one chunk as loaded (unconverted).  The gates of the next chunk are loaded into registers
    // one phase ahead (they are needed first); q, k and v of the next chunk are only touched (one 4-byte
    // read per 128-byte line) so that they wait in L2, and are loaded for real when the preparation starts:
    // holding all of them in registers across the contraction phases costs more registers than there are.
    struct RawG {
        Raw8<TG> g[RPT];
    };
    using RawV = typename std::conditional<kFull, Raw4<TIO>, Raw8<TIO>>::type;
    struct RawQKV {
        Raw8<TIO> q[kFull ? RPT : 1], k[RPT];
        RawV v[RPT];
    };
    struct Ptrs {   // uniform base pointers of the current chunk
        const TIO *q, *k, *v;
        const TG *g;
    };
    struct PrepAddr {   // per-lane LDS byte addresses used by prepare()
        uint32_t cs_w, cs_c, bc_w, bc_r, kt_w0, kt_w1, vt_w, qs_w;
    };

    // Tokens at or beyond `valid` read as zero (zero log-gate = no decay, zero k and v = no contribution).
    // A full chunk (valid == C, a workgroup-uniform condition) takes the branch without per-token tests.
    static __device__ __forceinline__ void load_gates(RawG &rg, const TG *gp, uint32_t rs, int valid, int sg,
                                                      uint32_t off)
    {
        if (valid >= C) {
#pragma unroll
            for (int j = 0; j < RPT; ++j) rg.g[j].load(gp + j * rs, off);
        } else {
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                if (sg * RPT + j < valid)
                    rg.g[j].load(gp + j * rs, off);
                else
                    rg.g[j].zero();
            }
        }
    }
    static __device__ __forceinline__ void load_qkv(RawQKV &rc, const Ptrs &p, uint32_t rs, int valid, int sg,
                                                    uint32_t off, uint32_t voff)
    {
        if (valid >= C) {
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                rc.k[j].load(p.k + j * rs, off);
                if (kFull) rc.q[j].load(p.q + j * rs, off);
                rc.v[j].load(p.v + j * rs, voff);
            }
        } else {
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                if (sg * RPT + j < valid) {
                    rc.k[j].load(p.k + j * rs, off);
                    if (kFull) rc.q[j].load(p.q + j * rs, off);
                    rc.v[j].load(p.v + j * rs, voff);
                } else {
                    rc.k[j].zero();
                    if (kFull) rc.q[j].zero();
                    rc.v[j].zero();
                }
            }
        }
    }
    // One 4-byte read per 128-byte line of the q, k, v rows of a chunk (rows below `valid` only).  The
    // value is returned so that the caller can keep it "in use" until the real loads have been issued.
    static constexpr int TOUCH_LPR = D * static_cast<int>(sizeof(TIO)) / 128;   // 128-byte lines per token row
    static constexpr int TOUCH_LPT = C * TOUCH_LPR;                             // lines per tensor and chunk
    static constexpr int TOUCH_NTEN = kFull ? 3 : 2;
    static constexpr int TOUCH_N = TOUCH_NTEN * ((TOUCH_LPT + NT - 1) / NT);    // touches per thread
    struct Touched {
        uint32_t x[TOUCH_N];
    };
    static __device__ __forceinline__ void touch_qkv(Touched &t, const Ptrs &p, uint32_t rs, int valid, int tid)
    {
        constexpr int PASSES = (TOUCH_LPT + NT - 1) / NT;
#pragma unroll
        for (int ten = 0; ten < TOUCH_NTEN; ++ten) {
            const TIO *tp = (ten == 0) ? p.k : (ten == 1) ? p.v : p.q;
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                // thread tid of pass ps touches line (ps * NT + tid) of every tensor
                const int l = ps * NT + tid;
                const int row = l / TOUCH_LPR, part = l % TOUCH_LPR;
                uint32_t x = 0;
                if (l < TOUCH_LPT && (valid >= C || row < valid)) {
                    const uint32_t boff = (static_cast<uint32_t>(row) * rs) * static_cast<uint32_t>(sizeof(TIO)) + part * 128;
                    x = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(tp) + boff);
                }
                t.x[ten * PASSES + ps] = x;
            }
        }
    }
    static __device__ __forceinline__ void touch_use(const Touched &t)
    {
#pragma unroll
        for (int i = 0; i < TOUCH_N; ++i) asm volatile("" ::"v"(t.x[i]));
    }

    // Per-lane LDS byte addresses of prepare().  They are derived inside the chunk loop from an opaque copy
    // of the thread index: a few integer operations per chunk instead of registers that would stay
    // occupied during the contraction phases.
    static __device__ __forceinline__ PrepAddr prep_addr(uint32_t sm, int ip, uint32_t u)   // ip: group index
    {
        const uint32_t dg = u % DG, sg = u / DG;
        PrepAddr pa;
        pa.cs_w = sm + CS + ((ip * SG + sg) * D + dg * 8) * 4;
        pa.cs_c = sm + CS + (ip * SG * D + u) * 4;
        pa.bc_w = sm + BC + (ip * D + u) * 4;
        pa.bc_r = sm + BC + (ip * D + dg * 8) * 4;
        const uint32_t r0 = ip * D + 16 * (dg >> 1) + 4 * (dg & 1), r1 = r0 + 8;
        pa.kt_w0 = sm + KT + (r0 * TP + tcol(r0, sg * RPT)) * ESZ;
        pa.kt_w1 = sm + KT + (r1 * TP + tcol(r1, sg * RPT)) * ESZ;
        const uint32_t rv = ip * (D / 2) + dg * VW;
        pa.vt_w = sm + VT + (rv * TP + tcol(rv, sg * RPT)) * ESZ;
        pa.qs_w = sm + QS + ((sg * RPT) * QP + ip * D + dg * 8) * ESZ;
        return pa;
    }

    // Cumulative natural-log gates over this thread's tokens, and the thread's total into the scan scratch.
    // Runs at the end of the previous chunk's iteration (before its output store), so that the gate
    // registers are consumed there and no load is waited for behind a store at the top of the loop.
    static __device__ __forceinline__ void gate_sums(float (&bl)[RPT][8], const RawG &rg, uint32_t cs_w)
    {
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            float g[8];
            rg.g[j].unpack(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) bl[j][e] = j ? bl[j - 1][e] + g[e] : g[e];
        }
        lds_st<f32x4>(cs_w, f32x4{bl[RPT - 1][0], bl[RPT - 1][1], bl[RPT - 1][2], bl[RPT - 1][3]});
        lds_st<f32x4>(cs_w + 16, f32x4{bl[RPT - 1][4], bl[RPT - 1][5], bl[RPT - 1][6], bl[RPT - 1][7]});
    }

    // Gate scan and operand preparation for one chunk.  Thread (ip, dg, sg) handles state ip, features
    // 8dg..8dg+7, tokens RPT*sg.. of q, k and the gate, and columns ip*D/2 + 4dg.. of v.  Ends with the
    // operands in LDS; the caller places the barrier.  lg = log2|gamma_ip scale|, neg = its sign.
    static __device__ __forceinline__ void prepare(const PrepAddr &pa, const float (&bl)[RPT][8], const RawQKV &rc,
                                                   float lg, bool neg, bool scans, float &seg_log2_decay,
                                                   PhaseClock &clk)
    {
        clk.mark(0);
        lds_barrier();
        clk.mark(1);
        if (scans) {   // thread u < D of a group scans feature u of its state over the token groups
            float t[SG];
#pragma unroll
            for (int s = 0; s < SG; ++s) t[s] = lds_ld<float>(pa.cs_c + s * D * 4);
            float run = 0.f;
#pragma unroll
            for (int s = 0; s < SG; ++s) {
                lds_st<float>(pa.cs_c + s * D * 4, run);
                run += t[s];
            }
            const float run2 = run * kLog2e;
            lds_st<float>(pa.bc_w, run2);
            lds_st<float>(pa.bc_w + (DEC - BC), __builtin_amdgcn_exp2f(run2));
            seg_log2_decay += run2;
        }
        lds_barrier();
        clk.mark(2);

        float pre2[8], bc[8];
        {
            const f32x4 p0 = lds_ld<f32x4>(pa.cs_w), p1 = lds_ld<f32x4>(pa.cs_w + 16);
            const f32x4 c0 = lds_ld<f32x4>(pa.bc_r), c1 = lds_ld<f32x4>(pa.bc_r + 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pre2[e] = p0[e] * kLog2e;   // log2 decay accumulated before this thread's first token
                pre2[4 + e] = p1[e] * kLog2e;
                bc[e] = c0[e];
                bc[4 + e] = c1[e];
            }
        }
        {   // ---- k: K^ = k 2^{bC - b} (token-contiguous) and K~ = K^ 2^{-bC} (row layout) ----
            float ak[8], einv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ak[e] = bc[e] - pre2[e];
                if (kFull) einv[e] = __builtin_amdgcn_exp2f(-bc[e]);
            }
            Row8 khat[RPT];
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                float kf[8], kh[8];
                rc.k[j].unpack(kf);
#pragma unroll
                for (int e = 0; e < 8; ++e) kh[e] = kf[e] * __builtin_amdgcn_exp2f(fmaf(bl[j][e], -kLog2e, ak[e]));
                khat[j] = A::pack_row(kh);
                if (kFull) {
                    float kt[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) kt[e] = kh[e] * einv[e];
                    A::store_row(pa.qs_w + (KS - QS) + j * QP * ESZ, A::pack_row(kt));
                }
                __builtin_amdgcn_sched_barrier(0);   // one token at a time: keeps the temporaries of a token short-lived
            }
            // rows rho(feature): e = 0..3 -> kt_w0 + e rows, e = 4..7 -> kt_w1 + (e - 4) rows
#pragma unroll
            for (int e = 0; e < 8; ++e)
                A::template store_tokens<RPT>((e < 4 ? pa.kt_w0 : pa.kt_w1) + (e & 3) * TP * ESZ, khat, e);
        }
        if (kFull) {   // ---- q: Q~ = gamma_i scale q 2^{b} (row layout) ----
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                float qf[8], qt[8];
                rc.q[j].unpack(qf);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    qt[e] = qf[e] * __builtin_amdgcn_exp2f(fmaf(bl[j][e], kLog2e, pre2[e] + lg));
                if (neg) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) qt[e] = -qt[e];
                }
                A::store_row(pa.qs_w + j * QP * ESZ, A::pack_row(qt));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // V transposed: this thread's VW columns (rows of Vt), RPT tokens each
#pragma unroll
        for (int e = 0; e < VW; ++e) store_v_tokens<RPT>(pa.vt_w + e * TP * ESZ, rc.v, e);
    }

    static __device__ void run(const PrefillArgs &a, uint32_t sm)
    {
        const int tid = threadIdx.x;
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, kept in scalar registers
        const int ln = lane & 31, g = lane >> 5;
        const int ct = wave % CT;                // column tile this wavefront owns in the contractions
        // Work item of the workgroup and state of this wavefront.  Chunk loop: block = (bh, segment), state =
        // wavefront group.  Pre-pass: block = (bh, segment, state); blocks 8 apart (same XCD, hence same L2
        // under round-robin dispatch) handle the two states of one (bh, segment) and share its k and v lines.
        const int nseg = kFull ? a.P : a.P - 1;
        int unit, ip;
        if (kFull) {
            unit = blockIdx.x;
            ip = wave / CT;
        } else {
            const int pairs = gridDim.x / 2;                      // (bh, segment) items
            const int blk = blockIdx.x, grp16 = blk / 16, in16 = blk % 16;
            if ((grp16 + 1) * 8 <= pairs) {                       // full 16-block group: 8 items x 2 states
                unit = grp16 * 8 + in16 % 8;
                ip = in16 / 8;
            } else {                                              // tail: adjacent blocks pair up
                const int rest = blk - grp16 * 16;
                unit = grp16 * 8 + rest / 2;
                ip = rest % 2;
            }
        }
        const int ipl = kFull ? ip : 0;          // group index inside the workgroup (LDS layout)
        const int u = tid - ipl * GT;            // index inside the group
        const int dg = u % DG, sg = u / DG;

        const int bh = unit / nseg;
        const int p = unit % nseg;
        const int bidx = bh / a.H, h = bh % a.H;
        const int BH = (kFull ? gridDim.x : gridDim.x / 2) / nseg;

        const int64_t t0 = static_cast<int64_t>(p) * a.seg_tokens;
        const int64_t t1 = (t0 + a.seg_tokens < a.T) ? t0 + a.seg_tokens : a.T;
        const uint32_t rs = static_cast<uint32_t>(a.H) * D;   // elements between consecutive tokens
        // uniform element offset of (b, t0, h, 0); per-lane offsets are 32-bit
        const size_t seg0 = (static_cast<size_t>(bidx) * a.T * a.H + h) * D + static_cast<size_t>(t0) * rs;
        // per-lane element offsets of the global accesses; evaluated from an opaque copy of the thread index
        // where they are used, so that they do not stay in registers across the other phases
        auto lane_off = [&](uint32_t uo) -> uint32_t { return (uo / DG) * RPT * rs + (uo % DG) * 8; };
        auto lane_voff = [&](uint32_t uo) -> uint32_t { return (uo / DG) * RPT * rs + ipl * (D / 2) + (uo % DG) * VW; };

        const float gm = a.gamma_per_head ? a.gamma_per_head[h] : a.gamma;
        const float gsv = (ip ? 1.0f - gm : gm) * a.scale;
        const float lg = __builtin_amdgcn_logf(fabsf(gsv));
        const bool neg = gsv < 0.f;

        // ---- state accumulators: tile dt covers Kt rows 32dt..32dt+31 of state ip, columns 32*ct.. ----
        // register j of lane (ln, g) holds state element (feature 32dt + 16(j/8) + 8g + j%8, column 32ct + ln)
        f32x16 acc[DT];
        const uint32_t sbase = static_cast<uint32_t>(8 * g) * D + 32 * ct + ln;  // lane part of the state offset
        if (kFull) {
            const float *src = (a.P > 1) ? a.ws_state + ((static_cast<size_t>(p) * BH + bh) * 2 + ip) * D * D
                                         : (ip ? a.S2 : a.S1) + static_cast<size_t>(bh) * D * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[dt][j] = src[sbase + (32 * dt + 16 * (j >> 3) + (j & 7)) * D];
        } else {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[dt][j] = 0.f;
        }

        const int own = (RT == 2) ? ip : 0;   // query tile this wavefront finishes
        // score tile of wavefronts 0..NTILE-1: RT = 1: (0,0); RT = 2: 0 -> (0,0), 1 -> (0,1), 2 -> (1,1)
        const int sc_ts = (RT == 2 && wave == 2) ? 1 : 0;
        const int sc_tr = (RT == 2 && wave >= 1) ? 1 : 0;

        float seg_decay = 0.f;  // threads u < D: log2 of the segment decay of feature u of state ip
        Ptrs ptr;
        ptr.q = static_cast<const TIO *>(a.q) + seg0;
        ptr.k = static_cast<const TIO *>(a.k) + seg0;
        ptr.g = static_cast<const TG *>(ip ? a.g2 : a.g1) + seg0;
        ptr.v = static_cast<const TIO *>(a.v) + seg0;
        TIO *optr = static_cast<TIO *>(a.o) + seg0;
        const size_t cstep = static_cast<size_t>(C) * rs;

        if (kFull && RT == 2) {
            // scores of keys 32..63 against queries 0..31 are in the future of every query: that block of As is
            // never computed; it is cleared once so that the read-out can run over all key blocks unconditionally
            for (int i = tid; i < 32 * 32 / 8; i += NT) {
                const int r = i / 4, c8 = i % 4;
                const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                A::store_row(sm + AS + (r * TP + 32 + 8 * c8) * ESZ, A::pack_row(z));
            }
        }
        RawG rg;
        int valid = (t1 - t0 >= C) ? C : static_cast<int>(t1 - t0);   // tokens of the current chunk
        load_gates(rg, ptr.g, rs, valid, sg, lane_off(u));
        Touched touched;
#pragma unroll
        for (int i = 0; i < TOUCH_N; ++i) touched.x[i] = 0;
        float bl[RPT][8];   // cumulative log-gates of the current chunk (computed one iteration ahead)
        gate_sums(bl, rg, sm + CS + ((ipl * SG + sg) * D + dg * 8) * 4);
        PhaseClock clk;
        clk.start();

        for (int64_t tc = t0; tc < t1; tc += C) {
            const bool has_next = tc + C < t1;
            const int64_t left_next = t1 - (tc + C);
            const int valid_next = has_next ? (left_next >= C ? C : static_cast<int>(left_next)) : 0;
            {
                // ---- this chunk's q/k/v: their lines wait in L2; first needed after the gate scan ----
                RawQKV rc;
                const uint32_t uo = opaque(static_cast<uint32_t>(u));
                load_qkv(rc, ptr, rs, valid, sg, lane_off(uo), lane_voff(uo));
                const PrepAddr pa = prep_addr(sm, ipl, uo);
                prepare(pa, bl, rc, lg, neg, u < D, seg_decay, clk);
            }
            clk.mark(3);
            lds_barrier();
            clk.mark(4);
            {
                // ---- next chunk: gates into registers (used at the end of this iteration) and one touch per
                //      line of its q/k/v rows, issued here where the memory pipeline is otherwise idle.  Past
                //      the end of the segment valid_next is 0: nothing is read and the gates become zeros. ----
                ptr.q += cstep; ptr.k += cstep; ptr.v += cstep; ptr.g += cstep;
                load_gates(rg, ptr.g, rs, valid_next, sg, lane_off(opaque(static_cast<uint32_t>(u))));
                if (!kFull) clk.mark(6);
                touch_qkv(touched, ptr, rs, valid_next, opaque(static_cast<uint32_t>(tid)));
                if (!kFull) clk.mark(8);
                valid = valid_next;
            }

            // ---- per-lane LDS addresses of the contraction phases (derived per chunk, see prep_addr) ----
            const uint32_t lq = opaque(static_cast<uint32_t>(lane));
            const uint32_t lnq = lq & 31, gq = lq >> 5;
            const uint32_t q_own = sm + QS + ((32 * own + lnq) * QP + ipl * D + 8 * gq) * ESZ;
            const uint32_t q_oth = sm + QS + ((32 * (RT - 1 - own) + lnq) * QP + ipl * D + 8 * gq) * ESZ;
            const uint32_t a_own = sm + AS + ((32 * own + lnq) * TP + 8 * gq) * ESZ;
            uint32_t vt_r[KB], kt_r[KB];   // swizzled token blocks of this lane's Vt row / first Kt row
            {
                const uint32_t vrow = 32 * ct + lnq, krow = ipl * D + lnq;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    vt_r[kb] = sm + VT + (vrow * TP + tcol(vrow, 16 * kb + 8 * gq)) * ESZ;
                    kt_r[kb] = sm + KT + (krow * TP + tcol(krow, 16 * kb + 8 * gq)) * ESZ;
                }
            }
            const uint32_t dec_r = sm + DEC + (ipl * D + 8 * gq) * 4;

            Frag sfr[kFull ? DT : 1][2];
            if (kFull && wave < NTILE) {
                // ---- scores, transposed: tile (ts, tr) holds S^T[s][r] for key tile ts <= query tile tr ----
                f32x16 sc;
#pragma unroll
                for (int j = 0; j < 16; ++j) sc[j] = 0.f;
                constexpr int NK = 2 * D / 16;
                // addresses used once per chunk are derived here from a per-iteration opaque copy of the lane
                // id, so that they do not occupy registers for the whole loop
                const uint32_t l2 = opaque(static_cast<uint32_t>(lane));
                const uint32_t lrow = (l2 & 31) * (QP * ESZ) + (l2 >> 5) * (8 * ESZ);
                const uint32_t sc_k = sm + KS + 32 * sc_ts * QP * ESZ + lrow;
                const uint32_t sc_q = sm + QS + 32 * sc_tr * QP * ESZ + lrow;
                const uint32_t sc_w =
                    sm + AS + (32 * sc_tr * TP + 32 * sc_ts) * ESZ + (l2 & 31) * (TP * ESZ) + (l2 >> 5) * (4 * ESZ);
                {
                    Frag held;   // the Ks fragment of a step waits here for its Qs partner
                    pipelined_steps<2 * NK, 8, A>(
                        [&](int s) -> uint32_t { return ((s & 1) ? sc_q : sc_k) + 16 * (s >> 1) * ESZ; },
                        [&](int s, const Frag &f) {
                            if ((s & 1) == 0)
                                held = f;
                            else
                                A::mma(sc, held, f);
                        });
                    // requested order: the fragment pairs of 4 steps are read ahead of the MFMAs
                    constexpr int RD = ESZ == 2 ? 1 : 2, MM = ESZ == 2 ? 1 : 8;
                    __builtin_amdgcn_sched_group_barrier(0x100, 8 * RD, 0);
#pragma unroll
                    for (int i = 0; i < NK - 4; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 2 * RD, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 4 * MM, 0);
                }
                // keep key <= query: key = 32 ts + 8 jb + 4 g + e, query = 32 tr + ln
                const int dq = 32 * (sc_tr - sc_ts) + ln - 4 * g;
#pragma unroll
                for (int jb = 0; jb < 4; ++jb) {
                    float x[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = (8 * jb + e <= dq) ? sc[4 * jb + e] : 0.f;
                    A::store4(sc_w + 8 * jb * ESZ, x[0], x[1], x[2], x[3]);
                }
            }
            // ---- carried state: take its input fragments for the read-out, then decay its rows.  The decay
            //      factors of two tiles (8 LDS reads) are requested together, ahead of the multiplies. ----
#pragma unroll
            for (int dt2 = 0; dt2 < DT; dt2 += 2) {
                constexpr int NTL = (DT >= 2) ? 2 : 1;   // tiles per batch
                f32x4 dd[NTL][4];
#pragma unroll
                for (int t = 0; t < NTL; ++t)
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb)
                        dd[t][jb] = lds_ld<f32x4>(dec_r + (32 * (dt2 + t) + 16 * (jb >> 1) + 4 * (jb & 1)) * 4);
                // all reads of the batch are in flight before the first one is consumed
                if constexpr (NTL == 2)
                    asm volatile("" : "+v"(dd[0][0]), "+v"(dd[0][1]), "+v"(dd[0][2]), "+v"(dd[0][3]), "+v"(dd[1][0]),
                                 "+v"(dd[1][1]), "+v"(dd[1][2]), "+v"(dd[1][3]));
                else
                    asm volatile("" : "+v"(dd[0][0]), "+v"(dd[0][1]), "+v"(dd[0][2]), "+v"(dd[0][3]));
#pragma unroll
                for (int t = 0; t < NTL; ++t) {
                    const int dt = dt2 + t;
                    if (kFull) {
                        sfr[dt][0] = A::from_acc(acc[dt], 0);
                        sfr[dt][1] = A::from_acc(acc[dt], 1);
                    }
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[dt][4 * jb + e] *= dd[t][jb][e];
                }
            }
            clk.mark(5);
            if (kFull) lds_barrier();
            clk.mark(6);

            // ---- V fragments of this wavefront's columns (input of both the output and the update) ----
            Frag vf[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) vf[kb] = A::load_frag(vt_r[kb]);

            // o_own: the query tile this wavefront finishes; o_oth: the tile the other group finishes (RT = 2)
            f32x16 o_own, o_oth;
            if (kFull) {
                // ---- partial output, transposed (o^T[column][query token]), summed over the features of
                //      state ip; the other group adds its state ----
#pragma unroll
                for (int j = 0; j < 16; ++j) o_own[j] = o_oth[j] = 0.f;
                {
                    constexpr int NS = DT * 2;   // steps over (dt, half): 16 features each
                    Frag f1 = A::load_frag(q_own), f2;
                    if (RT == 2) f2 = A::load_frag(q_oth);
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        const Frag c1 = f1, c2 = f2;
                        if (s + 1 < NS) {
                            f1 = A::load_frag(q_own + 16 * (s + 1) * ESZ);
                            if (RT == 2) f2 = A::load_frag(q_oth + 16 * (s + 1) * ESZ);
                        }
                        A::mma(o_own, sfr[s >> 1][s & 1], c1);
                        if (RT == 2) A::mma(o_oth, sfr[s >> 1][s & 1], c2);
                    }
                }
                // inside the chunk (key blocks in the future of the own query tile hold zeros)
                if (RT == 2 || ip == 0) {
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) A::mma(o_own, vf[kb], A::load_frag(a_own + 16 * kb * ESZ));
                }
                // hand over what the other group finishes: X[slot][jb][lane] (float4 units), in Ks
                const uint32_t x_w = sm + XB + (RT == 2 ? wave : ct) * 4096 + opaque(static_cast<uint32_t>(lane)) * 16;
                if (RT == 2) {
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb)
                        lds_st<f32x4>(x_w + jb * 1024,
                                      f32x4{o_oth[4 * jb], o_oth[4 * jb + 1], o_oth[4 * jb + 2], o_oth[4 * jb + 3]});
                } else if (ip == 1) {
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb)
                        lds_st<f32x4>(x_w + jb * 1024,
                                      f32x4{o_own[4 * jb], o_own[4 * jb + 1], o_own[4 * jb + 2], o_own[4 * jb + 3]});
                }
                if (RT == 2) {
                    // requested order for this region: LDS reads run 6 fragments ahead of the MFMAs
                    constexpr int RD = ESZ == 2 ? 1 : 2, MM = ESZ == 2 ? 1 : 8;
                    constexpr int NRD = KB + DT * 2 * RT + KB, NMM = DT * 2 * RT + KB;
                    __builtin_amdgcn_sched_group_barrier(0x100, 6 * RD, 0);
#pragma unroll
                    for (int i = 0; i < NRD - 6; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, (NMM - (NRD - 6)) * MM, 0);
                    __builtin_amdgcn_sched_group_barrier(0x200, 4, 0);
                }
            }

            clk.mark(7);
            if (kFull) {
                lds_barrier();
                clk.mark(8);
                // ---- finish the own output tile: own part + the other group's, staged in Qs ----
                if (RT == 2 || ip == 0) {
                    const uint32_t l2 = opaque(static_cast<uint32_t>(lane));
                    const uint32_t x_r = sm + XB + (RT == 2 ? (1 - ip) * CT + ct : ct) * 4096 + l2 * 16;
                    const uint32_t os_w =
                        sm + OS + (32 * own * OP + 32 * ct) * ESZ + (l2 & 31) * (OP * ESZ) + (l2 >> 5) * (4 * ESZ);
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb) {
                        const f32x4 x = lds_ld<f32x4>(x_r + jb * 1024);
                        A::store4(os_w + 8 * jb * ESZ, o_own[4 * jb] + x[0], o_own[4 * jb + 1] + x[1],
                                  o_own[4 * jb + 2] + x[2], o_own[4 * jb + 3] + x[3]);
                    }
                }
            }
            clk.mark(9);
            // ---- state update: add K^^T V to the decayed state.  Tile dt starts 32 dt rows further; the
            //      swizzle of odd tiles is that of even tiles with token blocks kb and kb^2 exchanged ----
            {
                constexpr int NS = KB * DT;
                auto kaddr = [&](int s) -> uint32_t {
                    const int dt = s % DT, kb = s / DT;
                    const int sw = (NC16 == 8) ? (kb ^ (2 * (dt & 1))) : kb;
                    return kt_r[sw] + 32 * dt * TP * ESZ;
                };
                pipelined_steps<NS, 4, A>(kaddr, [&](int s, const Frag &f) { A::mma(acc[s % DT], f, vf[s / DT]); });
                // requested instruction order for this region: LDS reads run 4 fragments ahead of the MFMAs
                constexpr int RD = ESZ == 2 ? 1 : 2;   // ds_read_b128 per fragment
                constexpr int MM = ESZ == 2 ? 1 : 8;   // MFMA instructions per fragment pair
                __builtin_amdgcn_sched_group_barrier(0x100, 4 * RD, 0);
#pragma unroll
                for (int s = 0; s < NS - 4; ++s) {
                    __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4 * MM, 0);
            }
            // ---- next chunk's gate sums: consumes the gates loaded at the top of this iteration, before the
            //      output store is issued (a wait for a load would otherwise also wait for the stores) ----
            {
                // The gates must not be consumed earlier than here (their load would be waited for right after it
                // was issued): the empty asm ties their registers to the last result of the update.
#pragma unroll
                for (int j = 0; j < RPT; ++j) rg.g[j].pin_after(acc[DT - 1][15]);
                const uint32_t uo = opaque(static_cast<uint32_t>(u));
                gate_sums(bl, rg, sm + CS + ((ipl * SG + uo / DG) * D + (uo % DG) * 8) * 4);
                touch_use(touched);
            }
            clk.mark(10);
            if (kFull) {
                lds_barrier();
                // ---- coalesced store of the staged output rows, 32 rows per pass ----
                const uint32_t t2 = opaque(static_cast<uint32_t>(tid));
                const uint32_t os_r = sm + OS + (t2 / DG) * (OP * ESZ) + (t2 % DG) * (8 * ESZ);
                const uint32_t ooff = (t2 / DG) * rs + (t2 % DG) * 8;   // 32 rows per pass
                const int64_t left = t1 - tc;
#pragma unroll
                for (int ps = 0; ps < RT; ++ps) {
                    if (32 * ps + static_cast<int>(t2 / DG) < left)
                        store8_global(optr + static_cast<size_t>(32 * ps) * rs, ooff, os_r + 32 * ps * OP * ESZ);
                }
                optr += cstep;
                clk.mark(11);
            }
            // The next prepare() writes Qs/Ks/Kt/Vt/dec only after its first scan barrier, which no
            // wavefront passes before every wavefront has finished the LDS reads above.
        }

#ifdef DSLA_PHASE_CLOCKS
        clk.flush(a.dbg);
#endif
        // ---- write the state out ----
        float *dst = nullptr;
        if (kFull) {
            if (p == a.P - 1) dst = (ip ? a.S2 : a.S1) + static_cast<size_t>(bh) * D * D;
        } else {
            // contribution of segment p goes to state slot p+1; its log2 decay to decay slot p
            dst = a.ws_state + ((static_cast<size_t>(p + 1) * BH + bh) * 2 + ip) * D * D;
            if (u < D) a.ws_decay[(static_cast<size_t>(p) * BH + bh) * 2 * D + ip * D + u] = seg_decay;
        }
        if (dst) {
            // recomputed on purpose (opaque): keeping the 16 DT offsets of the initial load alive across the
            // chunk loop would cost that many registers
            const uint32_t sb = opaque(static_cast<uint32_t>(8 * g) * D + 32 * ct + ln);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) dst[sb + (32 * dt + 16 * (j >> 3) + (j & 7)) * D] = acc[dt][j];
        }
    }
};

template <int D, int C, class TIO, class TG, bool kFull>
__global__ __launch_bounds__(kFull ? 4 * D : 2 * D, kFull ? 2 : 3) void prefill_kernel(PrefillArgs a)
{
    using K = Kern<D, C, TIO, TG, kFull>;
    __shared__ __attribute__((aligned(16))) char smem[K::LDS_BYTES];
    K::run(a, lds_addr_of(smem));
}

// Elementwise scan over segments: slot 0 <- caller's state; slot p+1 <- 2^{decay_p} * slot p + U_p,
// where U_p was left in slot p+1 by the segment_state kernel.
template <int D>
__global__ __launch_bounds__(256) void segment_scan_kernel(const float *__restrict__ S1, const float *__restrict__ S2,
                                                           float *__restrict__ ws_state,
                                                           const float *__restrict__ ws_decay, int BH, int P)
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
    const size_t bh = bi >> 1;
    const float *src = (i ? S2 : S1) + (bh * D + row) * D + c4 * 4;
    float4 s = *reinterpret_cast<const float4 *>(src);
    const size_t slot = static_cast<size_t>(BH) * 2 * D * D;
    float *w = ws_state + r * D + c4 * 4;
    *reinterpret_cast<float4 *>(w) = s;
    for (int p = 0; p + 1 < P; ++p) {
        const float dec = __builtin_amdgcn_exp2f(ws_decay[(static_cast<size_t>(p) * BH + bh) * 2 * D + i * D + row]);
        float4 *u = reinterpret_cast<float4 *>(w + static_cast<size_t>(p + 1) * slot);
        const float4 x = *u;
        s.x = fmaf(dec, s.x, x.x);
        s.y = fmaf(dec, s.y, x.y);
        s.z = fmaf(dec, s.z, x.z);
        s.w = fmaf(dec, s.w, x.w);
        *u = s;
    }
}

template <int D, int C, class TIO, class TG>
hipError_t launch_t(const dsla_desc &d, const PrefillPlan &plan, PrefillArgs &a, hipStream_t stream)
{
    const int BH = d.B * d.H;
    hipError_t err;
    if (plan.segments > 1) {
#ifdef DSLA_PHASE_CLOCKS
        static long long *dbg1 = nullptr;
        if (!dbg1) (void)hipMalloc(&dbg1, 16 * 12 * sizeof(long long));
        (void)hipMemsetAsync(dbg1, 0, 16 * 12 * sizeof(long long), stream);
        a.dbg = dbg1;
#endif
        {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_STATE, stream);
            hipLaunchKernelGGL((prefill_kernel<D, C, TIO, TG, false>), dim3(BH * (plan.segments - 1) * 2), dim3(2 * D),
                               0, stream, a);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
#ifdef DSLA_PHASE_CLOCKS
        {
            long long h[16 * 12];
            (void)hipStreamSynchronize(stream);
            (void)hipMemcpy(h, dbg1, sizeof(h), hipMemcpyDeviceToHost);
            for (int w = 0; w < 4 * D / 64; w += 4) {
                long long tot = 0;
                for (int n = 0; n < 12; ++n) tot += h[w * 12 + n];
                fprintf(stderr, "[segment_state clocks] wave %d total %lld:", w, tot);
                for (int n = 0; n < 12; ++n) fprintf(stderr, " %d=%lld", n, h[w * 12 + n]);
                fprintf(stderr, "\n");
            }
        }
#endif
        {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_SCAN, stream);
            const size_t n4 = static_cast<size_t>(BH) * 2 * D * (D / 4);
            hipLaunchKernelGGL((segment_scan_kernel<D>), dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0,
                               stream, a.S1, a.S2, a.ws_state, a.ws_decay, BH, plan.segments);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
    }
#ifdef DSLA_PHASE_CLOCKS
    static long long *dbg = nullptr;
    if (!dbg) (void)hipMalloc(&dbg, 16 * 12 * sizeof(long long));
    (void)hipMemsetAsync(dbg, 0, 16 * 12 * sizeof(long long), stream);
    a.dbg = dbg;
#endif
    {
        ProfileScope ps(DSLA_KERNEL_PREFILL_CHUNK_LOOP, stream);
        hipLaunchKernelGGL((prefill_kernel<D, C, TIO, TG, true>), dim3(BH * plan.segments), dim3(4 * D), 0, stream, a);
    }
    err = hipGetLastError();
#ifdef DSLA_PHASE_CLOCKS
    {
        long long h[16 * 12];
        (void)hipStreamSynchronize(stream);
        (void)hipMemcpy(h, dbg, sizeof(h), hipMemcpyDeviceToHost);
        static const char *names[12] = {"prep:cumsum", "prep:B1", "prep:scan+B2", "prep:operands", "loads+B3", "scores+state",
                                        "B4", "output", "B5", "finish", "loads+update", "B6+store"};
        for (int w = 0; w < 4 * D / 64; ++w) {
            long long tot = 0;
            for (int n = 0; n < 12; ++n) tot += h[w * 12 + n];
            fprintf(stderr, "[phase clocks] wave %d total %lld:", w, tot);
            for (int n = 0; n < 12; ++n) fprintf(stderr, " %s=%lld", names[n], h[w * 12 + n]);
            fprintf(stderr, "\n");
        }
    }
#endif
    return err;
}

template <int D, int C, class TIO>
hipError_t launch_g(const dsla_desc &d, const PrefillPlan &plan, PrefillArgs &a, hipStream_t stream)
{
    if (d.gate_dtype == DSLA_BF16) return launch_t<D, C, TIO, bf16_t>(d, plan, a, stream);
    return launch_t<D, C, TIO, float>(d, plan, a, stream);
}

bool combo_built(int D, int C, int io)
{
    if (io == DSLA_BF16) return (D == 64 || D == 128) && (C == 32 || C == 64);
    return (D == 64 && (C == 32 || C == 64)) || (D == 128 && C == 32);
}

}  // namespace

bool prefill_plan(const dsla_desc &d, int64_t T, PrefillPlan *plan)
{
    if (d.d_k != d.d_v) return false;
    const int D = d.d_k;
    int C = d.chunk;
    if (C == 0) C = combo_built(D, 64, d.io_dtype) ? 64 : 32;
    if (!combo_built(D, C, d.io_dtype)) return false;
    const int64_t nchunks = (T + C - 1) / C;
    const int64_t BH = static_cast<int64_t>(d.B) * d.H;
    int64_t P;
    if (d.segments > 0) {
        P = d.segments;
    } else {
        // enough workgroups to cover the 256 compute units (two per unit for the small head size),
        // but at least 4 chunks per segment so that the extra segment_state pass stays cheap
        const int64_t target = (D == 64) ? 512 : 256;
        P = target / BH;
        if (P > nchunks / 4) P = nchunks / 4;
    }
    if (P < 1) P = 1;
    if (P > nchunks) P = nchunks;
    const int64_t cps = (nchunks + P - 1) / P;
    P = (nchunks + cps - 1) / cps;
    plan->chunk = C;
    plan->segments = static_cast<int>(P);
    plan->segment_tokens = cps * C;
    plan->state_elems = static_cast<size_t>(BH) * D * D;
    if (P > 1) {
        plan->ws_state_bytes = static_cast<size_t>(P) * plan->state_elems * 2 * sizeof(float);
        plan->ws_decay_bytes = ((static_cast<size_t>(P - 1) * BH * 2 * D * sizeof(float)) + 255) / 256 * 256;
    } else {
        plan->ws_state_bytes = 0;
        plan->ws_decay_bytes = 0;
    }
    plan->ws_total_bytes = plan->ws_state_bytes + plan->ws_decay_bytes;
    return true;
}

hipError_t launch_prefill(const dsla_desc &d, const PrefillPlan &plan, int64_t T, const void *q, const void *k,
                          const void *v, const void *g1, const void *g2, float *S1, float *S2, void *o,
                          void *workspace, hipStream_t stream)
{
    PrefillArgs a;
    a.q = q; a.k = k; a.v = v; a.g1 = g1; a.g2 = g2; a.o = o;
    a.S1 = S1; a.S2 = S2;
    a.ws_state = static_cast<float *>(workspace);
    a.ws_decay = plan.segments > 1
                     ? reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.ws_state_bytes)
                     : nullptr;
    a.gamma_per_head = d.gamma_per_head;
    a.T = T;
    a.seg_tokens = plan.segment_tokens;
    a.H = d.H;
    a.P = plan.segments;
    a.gamma = d.gamma;
    a.scale = d.scale;
    const int D = d.d_k, C = plan.chunk;
    if (d.io_dtype == DSLA_BF16) {
        if (D == 128 && C == 64) return launch_g<128, 64, bf16_t>(d, plan, a, stream);
        if (D == 128 && C == 32) return launch_g<128, 32, bf16_t>(d, plan, a, stream);
        if (D == 64 && C == 64) return launch_g<64, 64, bf16_t>(d, plan, a, stream);
        if (D == 64 && C == 32) return launch_g<64, 32, bf16_t>(d, plan, a, stream);
    } else {
        if (D == 64 && C == 64) return launch_g<64, 64, float>(d, plan, a, stream);
        if (D == 64 && C == 32) return launch_g<64, 32, float>(d, plan, a, stream);
        if (D == 128 && C == 32) return launch_g<128, 32, float>(d, plan, a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace dsla
