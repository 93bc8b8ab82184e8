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
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// ---------------------------------------------------------------------------------------------
// Arithmetic-type policies: how a contraction operand is stored in LDS and fed to MFMA.
// A "fragment" is the 8 contraction-index values one lane supplies for a block of 16 contraction
// indices (lane group g = lane/32 supplies indices 8g..8g+7 of the block).
// ---------------------------------------------------------------------------------------------
struct ArithBf16 {
    using elem = uint16_t;  // LDS storage
    struct Frag {
        bf16x8 v;
    };
    struct Pack4 {
        uint2 v;
    };
    static __device__ __forceinline__ Frag load_frag(const elem *p)
    {
        const uint4 u = *reinterpret_cast<const uint4 *>(p);
        Frag f;
        f.v = __builtin_bit_cast(bf16x8, u);
        return f;
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        f32x2 x = {a, b};
        bf16x2 y = __builtin_convertvector(x, bf16x2);
        return __builtin_bit_cast(uint32_t, y);
    }
    static __device__ __forceinline__ void store4(elem *p, float a, float b, float c, float d)
    {
        *reinterpret_cast<uint2 *>(p) = make_uint2(pack2(a, b), pack2(c, d));
    }
    static __device__ __forceinline__ void store2(elem *p, float a, float b)
    {
        *reinterpret_cast<uint32_t *>(p) = pack2(a, b);
    }
    static __device__ __forceinline__ Frag from_acc(const f32x16 &acc, int half)
    {
        uint4 u;
        u.x = pack2(acc[8 * half + 0], acc[8 * half + 1]);
        u.y = pack2(acc[8 * half + 2], acc[8 * half + 3]);
        u.z = pack2(acc[8 * half + 4], acc[8 * half + 5]);
        u.w = pack2(acc[8 * half + 6], acc[8 * half + 7]);
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
    using elem = float;
    struct Frag {
        float v[8];
    };
    static __device__ __forceinline__ Frag load_frag(const elem *p)
    {
        const float4 a = *reinterpret_cast<const float4 *>(p);
        const float4 b = *reinterpret_cast<const float4 *>(p + 4);
        Frag f;
        f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
        f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
        return f;
    }
    static __device__ __forceinline__ void store4(elem *p, float a, float b, float c, float d)
    {
        *reinterpret_cast<float4 *>(p) = make_float4(a, b, c, d);
    }
    static __device__ __forceinline__ void store2(elem *p, float a, float b)
    {
        *reinterpret_cast<float2 *>(p) = make_float2(a, b);
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

// ---- raw 8-element global loads (kept unconverted while in flight) ----------------------------------
template <class T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
    uint4 u;
    __device__ __forceinline__ void load(const bf16_t *p) { u = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void zero() { u = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
        f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
        f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
        f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
    }
};
template <>
struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p)
    {
        a = *reinterpret_cast<const float4 *>(p);
        b = *reinterpret_cast<const float4 *>(p + 4);
    }
    __device__ __forceinline__ void zero() { a = b = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
};

__device__ __forceinline__ void store8_global(bf16_t *p, const uint16_t *lds8)
{
    *reinterpret_cast<uint4 *>(p) = *reinterpret_cast<const uint4 *>(lds8);
}
__device__ __forceinline__ void store8_global(float *p, const float *lds8)
{
    *reinterpret_cast<float4 *>(p) = *reinterpret_cast<const float4 *>(lds8);
    *reinterpret_cast<float4 *>(p + 4) = *reinterpret_cast<const float4 *>(lds8 + 4);
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
};

// Transposed store of V: element e of RPT consecutive tokens -> RPT adjacent LDS elements.
// bf16 data is moved with byte permutes (no conversion); fp32 data is stored as is.
template <int RPT>
__device__ __forceinline__ void store_v_tokens(uint16_t *dst, const Raw8<bf16_t> (&v)[RPT], int e)
{
    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
    auto word = [&](const uint4 &u) -> uint32_t {
        switch (e >> 1) {
        case 0: return u.x;
        case 1: return u.y;
        case 2: return u.z;
        default: return u.w;
        }
    };
    const uint32_t lo = __builtin_amdgcn_perm(word(v[1].u), word(v[0].u), sel);
    if (RPT == 4) {
        const uint32_t hi = __builtin_amdgcn_perm(word(v[3].u), word(v[2].u), sel);
        *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
    } else {
        *reinterpret_cast<uint32_t *>(dst) = lo;
    }
}
template <int RPT>
__device__ __forceinline__ void store_v_tokens(float *dst, const Raw8<float> (&v)[RPT], int e)
{
    auto pick = [&](const Raw8<float> &r) -> float {
        switch (e) {
        case 0: return r.a.x;
        case 1: return r.a.y;
        case 2: return r.a.z;
        case 3: return r.a.w;
        case 4: return r.b.x;
        case 5: return r.b.y;
        case 6: return r.b.z;
        default: return r.b.w;
        }
    };
    if (RPT == 4)
        *reinterpret_cast<float4 *>(dst) = make_float4(pick(v[0]), pick(v[1]), pick(v[2]), pick(v[3]));
    else
        *reinterpret_cast<float2 *>(dst) = make_float2(pick(v[0]), pick(v[1]));
}

template <int D, int C, class TIO, class TG, bool kFull>
struct Kern {
    using A = ArithOf<TIO>;
    using elem = typename A::elem;
    using Frag = typename A::Frag;

    static constexpr int NW = D / 32;       // wavefronts
    static constexpr int NT = 64 * NW;      // threads (= 2 D)
    static constexpr int DG = D / 8;        // feature groups of 8
    static constexpr int SG = NT / DG;      // token groups (16)
    static constexpr int RPT = C / SG;      // tokens per thread
    static constexpr int QP = 2 * D + 8;    // pitch of row-layout operands (elements)
    static constexpr int TP = C + 8;        // pitch of token-contiguous operands (elements)
    static constexpr int NC16 = C / 8;      // 8-element column groups in a token-contiguous row
    static constexpr int RT = C / 32;       // 32-token tiles in a chunk
    static constexpr int KB = C / 16;       // contraction blocks over tokens
    static constexpr int DT = D / 32;       // 32-row tiles of a state
    static_assert(SG == 16 && (RPT == 2 || RPT == 4), "chunk must be 32 or 64");
    static_assert(NT == 2 * D, "one thread per (state, feature) column in the gate scan");

    struct Smem {
        elem Qs[kFull ? C * QP : 8];    // [token][perm(i*D + d)]  gamma_i scale q 2^{b}
        elem Ks[kFull ? C * QP : 8];    // [token][perm(i*D + d)]  k 2^{-b}; reused as the o staging tile
        elem Kt[2 * D * TP];            // [i*D + d][token]        k 2^{bC - b}   (column groups swizzled)
        elem Vt[D * TP];                // [column][token]         v              (column groups swizzled)
        elem As[kFull ? C * TP : 8];    // [query token][key token] blended, masked scores
        float cs[SG * 2 * D];           // gate scan scratch: per token-group totals -> exclusive prefixes (ln)
        float bC[2 * D];                // log2 decay of the whole chunk, per (state, feature)
        float dec[2 * D];               // 2^{bC}
    };

    // swizzled offset inside a token-contiguous row: 8-element column group XOR (row / 8)
    static __device__ __forceinline__ int tcol(int row, int s)
    {
        return ((((s >> 3) ^ (row >> 3)) & (NC16 - 1)) << 3) | (s & 7);
    }

    struct RawChunk {
        Raw8<TIO> q[kFull ? RPT : 1], k[RPT], v[RPT];
        Raw8<TG> g1[RPT], g2[RPT];
    };

    // Per-thread global pointers at (first token this thread owns in the current chunk, feature group).
    struct Ptrs {
        const TIO *q, *k, *v;
        const TG *g1, *g2;
    };

    // Loads the tokens of one chunk this thread owns; tokens at or beyond `valid` read as zero
    // (zero log-gate = no decay, zero k and v = no contribution).
    static __device__ __forceinline__ void load_chunk(RawChunk &rc, const Ptrs &p, size_t rs, int valid, int sg)
    {
        if (valid >= C) {
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                if (kFull) rc.q[j].load(p.q + j * rs);
                rc.k[j].load(p.k + j * rs);
                rc.v[j].load(p.v + j * rs);
                rc.g1[j].load(p.g1 + j * rs);
                rc.g2[j].load(p.g2 + j * rs);
            }
        } else {
#pragma unroll
            for (int j = 0; j < RPT; ++j) {
                if (sg * RPT + j < valid) {
                    if (kFull) rc.q[j].load(p.q + j * rs);
                    rc.k[j].load(p.k + j * rs);
                    rc.v[j].load(p.v + j * rs);
                    rc.g1[j].load(p.g1 + j * rs);
                    rc.g2[j].load(p.g2 + j * rs);
                } else {
                    if (kFull) rc.q[j].zero();
                    rc.k[j].zero();
                    rc.v[j].zero();
                    rc.g1[j].zero();
                    rc.g2[j].zero();
                }
            }
        }
    }

    // Gate scan and operand preparation for one chunk (all threads).  Ends with the operands in LDS;
    // the caller places the barrier.  lg[i] = log2|gamma_i scale|, neg[i] = gamma_i scale < 0.
    static __device__ __forceinline__ void prepare(Smem &sm, const RawChunk &rc, const float (&lg)[2],
                                                   const bool (&neg)[2], int tid, float &seg_log2_decay)
    {
        const int dg = tid % DG, sg = tid / DG;
        float bl[2][RPT][8];  // cumulative natural-log gates over this thread's tokens
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            float g[8];
            rc.g1[j].unpack(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) bl[0][j][e] = j ? bl[0][j - 1][e] + g[e] : g[e];
            rc.g2[j].unpack(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) bl[1][j][e] = j ? bl[1][j - 1][e] + g[e] : g[e];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float *dst = &sm.cs[sg * 2 * D + i * D + dg * 8];
            *reinterpret_cast<float4 *>(dst) =
                make_float4(bl[i][RPT - 1][0], bl[i][RPT - 1][1], bl[i][RPT - 1][2], bl[i][RPT - 1][3]);
            *reinterpret_cast<float4 *>(dst + 4) =
                make_float4(bl[i][RPT - 1][4], bl[i][RPT - 1][5], bl[i][RPT - 1][6], bl[i][RPT - 1][7]);
        }
        lds_barrier();
        {   // thread c scans column c = (state, feature) over the token groups
            float t[SG];
#pragma unroll
            for (int s = 0; s < SG; ++s) t[s] = sm.cs[s * 2 * D + tid];
            float run = 0.f;
#pragma unroll
            for (int s = 0; s < SG; ++s) {
                sm.cs[s * 2 * D + tid] = run;
                run += t[s];
            }
            const float run2 = run * kLog2e;
            sm.bC[tid] = run2;
            sm.dec[tid] = __builtin_amdgcn_exp2f(run2);
            seg_log2_decay += run2;
        }
        lds_barrier();

        float kf[RPT][8];
#pragma unroll
        for (int j = 0; j < RPT; ++j) rc.k[j].unpack(kf[j]);

#pragma unroll
        for (int i = 0; i < 2; ++i) {
            float aq[8], ak[8], einv[8];
            {
                const float *src = &sm.cs[sg * 2 * D + i * D + dg * 8];
                const float4 p0 = *reinterpret_cast<const float4 *>(src);
                const float4 p1 = *reinterpret_cast<const float4 *>(src + 4);
                const float *sb = &sm.bC[i * D + dg * 8];
                const float4 c0 = *reinterpret_cast<const float4 *>(sb);
                const float4 c1 = *reinterpret_cast<const float4 *>(sb + 4);
                const float pre[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                const float bc[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float p2 = pre[e] * kLog2e;
                    aq[e] = p2 + lg[i];    // exponent of gamma_i scale 2^{b}: add the local part
                    ak[e] = bc[e] - p2;    // exponent of 2^{bC - b}: subtract the local part
                    if (kFull) einv[e] = __builtin_amdgcn_exp2f(-bc[e]);
                }
            }
            float khat[RPT][8];
#pragma unroll
            for (int j = 0; j < RPT; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    khat[j][e] = kf[j][e] * __builtin_amdgcn_exp2f(fmaf(bl[i][j][e], -kLog2e, ak[e]));
            // K^ transposed: row = i*D + feature, RPT consecutive tokens per store
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int row = i * D + dg * 8 + e;
                elem *dst = &sm.Kt[row * TP + tcol(row, sg * RPT)];
                if (RPT == 4)
                    A::store4(dst, khat[0][e], khat[1][e], khat[2][e], khat[3][e]);
                else
                    A::store2(dst, khat[0][e], khat[1][e]);
            }
            if (kFull) {
                // position of this thread's 8 features inside a permuted row: two groups of 4
                const int p0 = i * D + (dg >> 1) * 16 + (dg & 1) * 4;
#pragma unroll
                for (int j = 0; j < RPT; ++j) {
                    float qf[8];
                    rc.q[j].unpack(qf);
                    float qt[8], kt[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float eq = __builtin_amdgcn_exp2f(fmaf(bl[i][j][e], kLog2e, aq[e]));
                        if (neg[i]) eq = -eq;
                        qt[e] = qf[e] * eq;
                        kt[e] = khat[j][e] * einv[e];
                    }
                    const int row = sg * RPT + j;
                    A::store4(&sm.Qs[row * QP + p0], qt[0], qt[1], qt[2], qt[3]);
                    A::store4(&sm.Qs[row * QP + p0 + 8], qt[4], qt[5], qt[6], qt[7]);
                    A::store4(&sm.Ks[row * QP + p0], kt[0], kt[1], kt[2], kt[3]);
                    A::store4(&sm.Ks[row * QP + p0 + 8], kt[4], kt[5], kt[6], kt[7]);
                }
            }
        }
        // V transposed
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int row = dg * 8 + e;
            store_v_tokens<RPT>(&sm.Vt[row * TP + tcol(row, sg * RPT)], rc.v, e);
        }
    }

    // accumulator register j of a 32x32 tile holds tile row 8*(j/4) + 4*g + (j%4), tile column lane%32
    static __device__ __forceinline__ int acc_row(int j, int g) { return 8 * (j >> 2) + 4 * g + (j & 3); }

    static __device__ void run(const PrefillArgs &a, Smem &sm)
    {
        const int tid = threadIdx.x;
        const int lane = tid & 63, wave = tid >> 6;
        const int ln = lane & 31, g = lane >> 5;
        const int dg = tid % DG, sg = tid / DG;

        const int nseg = kFull ? a.P : a.P - 1;
        const int bh = blockIdx.x / nseg;
        const int p = blockIdx.x % nseg;
        const int bidx = bh / a.H, h = bh % a.H;
        const int BH = gridDim.x / nseg;

        const int64_t t0 = static_cast<int64_t>(p) * a.seg_tokens;
        const int64_t t1 = (t0 + a.seg_tokens < a.T) ? t0 + a.seg_tokens : a.T;
        const size_t rs = static_cast<size_t>(a.H) * D;
        // element offset of (b, first token this thread owns, h, feature group)
        const size_t off0 = (static_cast<size_t>(bidx) * a.T * a.H + h) * D +
                            static_cast<size_t>(t0 + sg * RPT) * rs + dg * 8;

        const float gm = a.gamma_per_head ? a.gamma_per_head[h] : a.gamma;
        const float gsv[2] = {gm * a.scale, (1.0f - gm) * a.scale};
        const float lg[2] = {__builtin_amdgcn_logf(fabsf(gsv[0])), __builtin_amdgcn_logf(fabsf(gsv[1]))};
        const bool neg[2] = {gsv[0] < 0.f, gsv[1] < 0.f};

        // ---- state accumulators: tile (i, dt) covers rows 32dt..32dt+31 of state i, columns 32*wave.. ----
        f32x16 acc[2][DT];
        const int col = 32 * wave + ln;
        if (kFull) {
            const float *src1 = (a.P > 1) ? a.ws_state + ((static_cast<size_t>(p) * BH + bh) * 2 + 0) * D * D
                                          : a.S1 + static_cast<size_t>(bh) * D * D;
            const float *src2 = (a.P > 1) ? a.ws_state + ((static_cast<size_t>(p) * BH + bh) * 2 + 1) * D * D
                                          : a.S2 + static_cast<size_t>(bh) * D * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int row = 32 * dt + acc_row(j, g);
                    acc[0][dt][j] = src1[static_cast<size_t>(row) * D + col];
                    acc[1][dt][j] = src2[static_cast<size_t>(row) * D + col];
                }
        } else {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[0][dt][j] = acc[1][dt][j] = 0.f;
        }

        float seg_decay = 0.f;  // thread tid: log2 of the segment decay of (state, feature) column tid
        Ptrs ptr;
        ptr.q = static_cast<const TIO *>(a.q) + off0;
        ptr.k = static_cast<const TIO *>(a.k) + off0;
        ptr.v = static_cast<const TIO *>(a.v) + off0;
        ptr.g1 = static_cast<const TG *>(a.g1) + off0;
        ptr.g2 = static_cast<const TG *>(a.g2) + off0;
        TIO *optr = static_cast<TIO *>(a.o) + off0;
        const size_t cstep = static_cast<size_t>(C) * rs;

        RawChunk rc;
        {
            const int64_t left = t1 - t0;
            load_chunk(rc, ptr, rs, left >= C ? C : static_cast<int>(left), sg);
        }

        for (int64_t tc = t0; tc < t1; tc += C) {
            prepare(sm, rc, lg, neg, tid, seg_decay);
            ptr.q += cstep; ptr.k += cstep; ptr.v += cstep; ptr.g1 += cstep; ptr.g2 += cstep;
            if (tc + C < t1) {  // next chunk: in flight during the contractions
                const int64_t left = t1 - (tc + C);
                load_chunk(rc, ptr, rs, left >= C ? C : static_cast<int>(left), sg);
            }
            lds_barrier();

            Frag sfr[kFull ? 2 : 1][kFull ? DT : 1][2];
            if (kFull) {
                // ---- scores, transposed: tile (ts, tr) holds S^T[s][r] for key tile ts <= query tile tr ----
                constexpr int NTILE = RT * (RT + 1) / 2;
#pragma unroll
                for (int tt = 0; tt < NTILE; ++tt) {
                    if (tt % NW != wave) continue;
                    // enumerate (ts, tr), ts <= tr: RT = 1: (0,0); RT = 2: (0,0) (0,1) (1,1)
                    const int ts = (RT == 2 && tt == 2) ? 1 : 0;
                    const int tr = (RT == 2 && tt >= 1) ? 1 : 0;
                    f32x16 sc;
#pragma unroll
                    for (int j = 0; j < 16; ++j) sc[j] = 0.f;
                    const elem *kp = &sm.Ks[(32 * ts + ln) * QP + 8 * g];
                    const elem *qp = &sm.Qs[(32 * tr + ln) * QP + 8 * g];
#pragma unroll
                    for (int kb = 0; kb < 2 * D / 16; ++kb) {
                        const Frag fa = A::load_frag(kp + 16 * kb);
                        const Frag fb = A::load_frag(qp + 16 * kb);
                        A::mma(sc, fa, fb);
                    }
                    const int r = 32 * tr + ln;
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb) {
                        const int s0 = 32 * ts + 8 * jb + 4 * g;
                        float x[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) x[e] = (s0 + e <= r) ? sc[4 * jb + e] : 0.f;
                        A::store4(&sm.As[r * TP + s0], x[0], x[1], x[2], x[3]);
                    }
                }
            }
            // ---- carried state: take its input fragments for the read-out, then decay its rows ----
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    if (kFull) {
                        sfr[i][dt][0] = A::from_acc(acc[i][dt], 0);
                        sfr[i][dt][1] = A::from_acc(acc[i][dt], 1);
                    }
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb) {
                        const float4 dd = *reinterpret_cast<const float4 *>(&sm.dec[i * D + 32 * dt + 8 * jb + 4 * g]);
                        acc[i][dt][4 * jb + 0] *= dd.x;
                        acc[i][dt][4 * jb + 1] *= dd.y;
                        acc[i][dt][4 * jb + 2] *= dd.z;
                        acc[i][dt][4 * jb + 3] *= dd.w;
                    }
                }
            if (kFull) lds_barrier();

            // ---- V fragments of this wavefront's columns (input of both the output and the update) ----
            Frag vf[KB];
            {
                const int row = 32 * wave + ln;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) vf[kb] = A::load_frag(&sm.Vt[row * TP + tcol(row, 16 * kb + 8 * g)]);
            }

            if (kFull) {
                // ---- output, transposed: tile tr holds o^T[column][query token] ----
                f32x16 oacc[RT];
#pragma unroll
                for (int tr = 0; tr < RT; ++tr)
#pragma unroll
                    for (int j = 0; j < 16; ++j) oacc[tr][j] = 0.f;
                // inside the chunk: sum over key tokens (blocks wholly in the future of a query tile are zero)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int tr = 0; tr < RT; ++tr) {
                        if (16 * kb > 32 * tr + 31) continue;
                        const Frag fb = A::load_frag(&sm.As[(32 * tr + ln) * TP + 16 * kb + 8 * g]);
                        A::mma(oacc[tr], vf[kb], fb);
                    }
                // carried state: the fragments taken from the accumulators are the other input
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int kpos = i * D + 32 * dt + 16 * half + 8 * g;
#pragma unroll
                            for (int tr = 0; tr < RT; ++tr) {
                                const Frag fb = A::load_frag(&sm.Qs[(32 * tr + ln) * QP + kpos]);
                                A::mma(oacc[tr], sfr[i][dt][half], fb);
                            }
                        }
                // stage o (Ks is free since the scores barrier): Os[token][column], pitch D + 8
                elem *Os = sm.Ks;
#pragma unroll
                for (int tr = 0; tr < RT; ++tr)
#pragma unroll
                    for (int jb = 0; jb < 4; ++jb) {
                        const int c0 = 32 * wave + 8 * jb + 4 * g;
                        A::store4(&Os[(32 * tr + ln) * (D + 8) + c0], oacc[tr][4 * jb + 0], oacc[tr][4 * jb + 1],
                                  oacc[tr][4 * jb + 2], oacc[tr][4 * jb + 3]);
                    }
            }

            // ---- state update: add K^^T V to the decayed state ----
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const int row = i * D + 32 * dt + ln;
                        const Frag fa = A::load_frag(&sm.Kt[row * TP + tcol(row, 16 * kb + 8 * g)]);
                        A::mma(acc[i][dt], fa, vf[kb]);
                    }

            if (kFull) {
                lds_barrier();
                // ---- coalesced store of the staged output rows ----
                const elem *Os = sm.Ks;
                const int64_t left = t1 - tc;
#pragma unroll
                for (int j = 0; j < RPT; ++j) {
                    const int r = sg * RPT + j;
                    if (r < left) store8_global(optr + j * rs, &Os[r * (D + 8) + dg * 8]);
                }
                optr += cstep;
            }
            // The next prepare() writes Qs/Ks/Kt/Vt/dec only after its first scan barrier, which no
            // wavefront passes before every wavefront has finished the LDS reads above.
        }

        // ---- write the state out ----
        if (kFull) {
            if (p == a.P - 1) {
                float *d1 = a.S1 + static_cast<size_t>(bh) * D * D;
                float *d2 = a.S2 + static_cast<size_t>(bh) * D * D;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int row = 32 * dt + acc_row(j, g);
                        d1[static_cast<size_t>(row) * D + col] = acc[0][dt][j];
                        d2[static_cast<size_t>(row) * D + col] = acc[1][dt][j];
                    }
            }
        } else {
            // contribution of segment p goes to state slot p+1; its log2 decay to decay slot p
            float *d1 = a.ws_state + ((static_cast<size_t>(p + 1) * BH + bh) * 2 + 0) * D * D;
            float *d2 = d1 + static_cast<size_t>(D) * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int row = 32 * dt + acc_row(j, g);
                    d1[static_cast<size_t>(row) * D + col] = acc[0][dt][j];
                    d2[static_cast<size_t>(row) * D + col] = acc[1][dt][j];
                }
            a.ws_decay[(static_cast<size_t>(p) * BH + bh) * 2 * D + tid] = seg_decay;
        }
    }
};

template <int D, int C, class TIO, class TG, bool kFull>
__global__ __launch_bounds__(2 * D) void prefill_kernel(PrefillArgs a)
{
    using K = Kern<D, C, TIO, TG, kFull>;
    __shared__ __attribute__((aligned(16))) typename K::Smem sm;
    K::run(a, sm);
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
        {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_STATE, stream);
            hipLaunchKernelGGL((prefill_kernel<D, C, TIO, TG, false>), dim3(BH * (plan.segments - 1)), dim3(2 * D), 0,
                               stream, a);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
        {
            ProfileScope ps(DSLA_KERNEL_PREFILL_SEGMENT_SCAN, stream);
            const size_t n4 = static_cast<size_t>(BH) * 2 * D * (D / 4);
            hipLaunchKernelGGL((segment_scan_kernel<D>), dim3(static_cast<unsigned>((n4 + 255) / 256)), dim3(256), 0,
                               stream, a.S1, a.S2, a.ws_state, a.ws_decay, BH, plan.segments);
            err = hipGetLastError();
        }
        if (err != hipSuccess) return err;
    }
    ProfileScope ps(DSLA_KERNEL_PREFILL_CHUNK_LOOP, stream);
    hipLaunchKernelGGL((prefill_kernel<D, C, TIO, TG, true>), dim3(BH * plan.segments), dim3(2 * D), 0, stream, a);
    return hipGetLastError();
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
