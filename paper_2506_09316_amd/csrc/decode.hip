// Fused DSLA decode step (paper Section 4.1: state-update equation and blended read-out,
// applied to one token per sequence).
//
// Bandwidth-bound: per (batch, head) the two fp32 states (2 * d_k * d_v * 4 bytes) are read
// once and written once; everything else is a few hundred bytes.  SPLIT workgroups of 256
// threads stream one (batch, head) pair, each a slice of the columns (the read-out of a column
// needs no other column).  A thread owns four adjacent state columns
// (one 16-byte access) in every ROWG-th row, so a wavefront access covers whole rows and is
// fully coalesced.  All state loads are issued before anything else so that the maximum
// number of bytes is in flight; the small per-token vectors go through LDS meanwhile.
#include "dsla_internal.h"

namespace dsla {
namespace {

constexpr int kDecodeThreads = 256;

// A state row piece as a streaming (non-temporal) load: a state is read once per step and written back, and the
// next read of it is a whole batch later; kept out of the caches' allocation the reads run 2 % faster
// (106.6 -> 104.3 us per step at B = 64).  The stores stay ordinary: streaming stores measured slower.
__device__ __forceinline__ float4 load_streaming(const float4 *p)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 x = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
    return make_float4(x[0], x[1], x[2], x[3]);
}

template <int DK, int DV, int SPLIT, class TIO, class TG>
__global__ __launch_bounds__(kDecodeThreads) void decode_kernel(
    const TIO *__restrict__ q, const TIO *__restrict__ k, const TIO *__restrict__ v, const TG *__restrict__ g1,
    const TG *__restrict__ g2, const int32_t *__restrict__ row, const int32_t *__restrict__ slot,
    float *__restrict__ S1, float *__restrict__ S2, TIO *__restrict__ o, int H, float gamma, const float *__restrict__ gamma_per_head, float scale, float gate_inv_tau)
{
    constexpr int COLG = DV / 4 / SPLIT;          // threads across this workgroup's part of a state row (float4 each)
    constexpr int ROWG = kDecodeThreads / COLG;   // row groups
    constexpr int ROWS = DK / ROWG;               // rows per thread
    static_assert(kDecodeThreads % COLG == 0 && DK % ROWG == 0, "shape");
    static_assert(COLG <= 64 && 64 % COLG == 0, "a wavefront must hold whole row groups");

    __shared__ float s_q[DK], s_k[DK], s_a1[DK], s_a2[DK];
    __shared__ float4 s_red[kDecodeThreads / 64][COLG];

    const int bh = blockIdx.x / SPLIT;
    const int part = blockIdx.x % SPLIT;          // which slice of the columns
    const int tid = threadIdx.x;
    const int cg = tid % COLG;
    const int rg = tid / COLG;
    constexpr int ROWF4 = DV / 4;                 // float4 per state row
    // the states of sequence b live in entry slot[b] of the state arrays (entry b without a slot list)
    const size_t sbase = (slot ? static_cast<size_t>(slot[bh / H]) * H + bh % H : static_cast<size_t>(bh)) * DK * DV;
    float4 *p1 = reinterpret_cast<float4 *>(S1 + sbase) + part * COLG + cg;
    float4 *p2 = reinterpret_cast<float4 *>(S2 + sbase) + part * COLG + cg;

    // 1. all state loads in flight
    float4 a[ROWS], b[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const int row = rg + j * ROWG;
        a[j] = load_streaming(&p1[static_cast<size_t>(row) * ROWF4]);
        b[j] = load_streaming(&p2[static_cast<size_t>(row) * ROWF4]);
    }

    // 2. per-token vectors -> LDS (gates exponentiated once per row)
    const float gm = gamma_per_head ? gamma_per_head[bh % H] : gamma;
    // the token of sequence b sits in row row[b] of q, k, v, g1, g2 and o (row b without a row list)
    const size_t tbh = row ? static_cast<size_t>(row[bh / H]) * H + bh % H : static_cast<size_t>(bh);
    const size_t kb = tbh * DK;
    for (int d = tid; d < DK; d += kDecodeThreads) {
        s_q[d] = scale * to_f32(q[kb + d]);
        s_k[d] = to_f32(k[kb + d]);
        float x1 = to_f32(g1[kb + d]), x2 = to_f32(g2[kb + d]);
        if (gate_inv_tau != 0.f) {   // pre-activations: log(sigmoid(z)^(1/tau)) = (min(z, 0) - log(1 + e^-|z|)) / tau
            x1 = (fminf(x1, 0.f) - log1pf(expf(-fabsf(x1)))) * gate_inv_tau;
            x2 = (fminf(x2, 0.f) - log1pf(expf(-fabsf(x2)))) * gate_inv_tau;
        }
        s_a1[d] = __expf(x1);
        s_a2[d] = __expf(x2);
    }
    const TIO *vp = v + tbh * DV + (part * COLG + cg) * 4;
    const float v0 = to_f32(vp[0]), v1 = to_f32(vp[1]), v2 = to_f32(vp[2]), v3 = to_f32(vp[3]);
    __syncthreads();

    // 3. update both states, accumulate the read-out, store
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const float gm2 = 1.0f - gm;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const int row = rg + j * ROWG;
        const float a1 = s_a1[row], a2 = s_a2[row], kd = s_k[row], qd = s_q[row];
        float4 x = a[j], y = b[j];
        x.x = fmaf(a1, x.x, kd * v0); x.y = fmaf(a1, x.y, kd * v1);
        x.z = fmaf(a1, x.z, kd * v2); x.w = fmaf(a1, x.w, kd * v3);
        y.x = fmaf(a2, y.x, kd * v0); y.y = fmaf(a2, y.y, kd * v1);
        y.z = fmaf(a2, y.z, kd * v2); y.w = fmaf(a2, y.w, kd * v3);
        p1[static_cast<size_t>(row) * ROWF4] = x;
        p2[static_cast<size_t>(row) * ROWF4] = y;
        const float qa = qd * gm, qb = qd * gm2;
        acc.x = fmaf(qa, x.x, fmaf(qb, y.x, acc.x));
        acc.y = fmaf(qa, x.y, fmaf(qb, y.y, acc.y));
        acc.z = fmaf(qa, x.z, fmaf(qb, y.z, acc.z));
        acc.w = fmaf(qa, x.w, fmaf(qb, y.w, acc.w));
    }

    // 4. reduce the read-out over row groups: inside a wavefront by shuffles, across by LDS
#pragma unroll
    for (int off = 32; off >= COLG; off >>= 1) {
        acc.x += __shfl_xor(acc.x, off);
        acc.y += __shfl_xor(acc.y, off);
        acc.z += __shfl_xor(acc.z, off);
        acc.w += __shfl_xor(acc.w, off);
    }
    const int wave = tid / 64, lane = tid % 64;
    if (lane < COLG) s_red[wave][lane] = acc;
    __syncthreads();
    if (tid < COLG) {
        float4 r = s_red[0][tid];
#pragma unroll
        for (int w = 1; w < kDecodeThreads / 64; ++w) {
            const float4 t = s_red[w][tid];
            r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w;
        }
        TIO *op = o + tbh * DV + (part * COLG + tid) * 4;
        op[0] = from_f32<TIO>(r.x);
        op[1] = from_f32<TIO>(r.y);
        op[2] = from_f32<TIO>(r.z);
        op[3] = from_f32<TIO>(r.w);
    }
}

// The decode step with N states, the outer-product gate and grouped key/value heads (background section on gated
// linear attention; Section 4.2; the state-count ablation of Section 5.5): per state n
//     S^n[d][j] <- alpha^n[d] beta^n[j] S^n[d][j] + k[d] v[j],       o[j] = scale sum_d q[d] sum_n w_n S^n[d][j].
// Same streaming pattern as decode_kernel; the states are taken one after the other, the loads of the next state in
// flight while the current one is updated, so every state is still read once and written once.
template <int DK, int DV, int SPLIT, class TIO, class TG>
__global__ __launch_bounds__(kDecodeThreads) void decode_multi_kernel(
    const TIO *__restrict__ q, const TIO *__restrict__ k, const TIO *__restrict__ v, MultiStatePtrs mp, int N,
    const int32_t *__restrict__ row, const int32_t *__restrict__ slot, TIO *__restrict__ o, int H, int Hkv,
    const float *__restrict__ w_per_head, float scale, float gate_inv_tau)
{
    constexpr int COLG = DV / 4 / SPLIT;
    constexpr int ROWG = kDecodeThreads / COLG;
    constexpr int ROWS = DK / ROWG;
    constexpr int ROWF4 = DV / 4;
    constexpr int NMAX = DSLA_MAX_STATES;
    __shared__ float s_q[DK], s_k[DK], s_alpha[NMAX][DK], s_beta[NMAX][COLG * 4], s_w[NMAX];
    __shared__ float4 s_red[kDecodeThreads / 64][COLG];

    const int bh = blockIdx.x / SPLIT;
    const int part = blockIdx.x % SPLIT;
    const int tid = threadIdx.x;
    const int cg = tid % COLG;
    const int rg = tid / COLG;
    const int b = bh / H, h = bh % H;
    const size_t sbase = ((slot ? static_cast<size_t>(slot[b]) : static_cast<size_t>(b)) * H + h) * DK * DV;
    const size_t c4 = static_cast<size_t>(part) * COLG + cg;   // this thread's float4 inside a state row

    auto load_state = [&](int n, float4 (&x)[ROWS]) {
        const float4 *p = reinterpret_cast<const float4 *>(mp.S[n] + sbase) + c4;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) x[j] = load_streaming(&p[static_cast<size_t>(rg + j * ROWG) * ROWF4]);
    };
    float4 cur[ROWS], nxt[ROWS];
    load_state(0, cur);

    // per-token vectors -> LDS: q, k once, the gates of every state
    const size_t trow = row ? static_cast<size_t>(row[b]) : static_cast<size_t>(b);
    const size_t tq = (trow * H + h) * DK;                         // q, alpha gates
    const size_t tk = (trow * Hkv + h / (H / Hkv)) * DK;           // k: the key/value head of this group
    auto log_gate = [&](float x) -> float {
        if (gate_inv_tau != 0.f) x = (fminf(x, 0.f) - log1pf(expf(-fabsf(x)))) * gate_inv_tau;
        return x;
    };
    for (int d = tid; d < DK; d += kDecodeThreads) {
        s_q[d] = scale * to_f32(q[tq + d]);
        s_k[d] = to_f32(k[tk + d]);
    }
    for (int i = tid; i < N * DK; i += kDecodeThreads) {
        const int n = i / DK, d = i % DK;
        s_alpha[n][d] = __expf(log_gate(to_f32(static_cast<const TG *>(mp.ga[n])[tq + d])));
    }
    for (int i = tid; i < N * COLG * 4; i += kDecodeThreads) {
        const int n = i / (COLG * 4), c = i % (COLG * 4);
        const size_t col = (trow * H + h) * DV + part * COLG * 4 + c;
        s_beta[n][c] = mp.gb[n] ? __expf(log_gate(to_f32(static_cast<const TG *>(mp.gb[n])[col]))) : 1.0f;
    }
    if (tid < N) s_w[tid] = w_per_head ? w_per_head[static_cast<size_t>(tid) * H + h] : mp.w[tid];
    const TIO *vp = v + (trow * Hkv + h / (H / Hkv)) * DV + c4 * 4;
    const float v0 = to_f32(vp[0]), v1 = to_f32(vp[1]), v2 = to_f32(vp[2]), v3 = to_f32(vp[3]);
    __syncthreads();

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int n = 0; n < N; ++n) {
        if (n + 1 < N) load_state(n + 1, nxt);
        float4 *p = reinterpret_cast<float4 *>(mp.S[n] + sbase) + c4;
        const float b0 = s_beta[n][cg * 4 + 0], b1 = s_beta[n][cg * 4 + 1], b2 = s_beta[n][cg * 4 + 2],
                    b3 = s_beta[n][cg * 4 + 3];
        const float wn = s_w[n];
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const int r = rg + j * ROWG;
            const float a = s_alpha[n][r], kd = s_k[r], qw = s_q[r] * wn;
            float4 x = cur[j];
            x.x = fmaf(a * b0, x.x, kd * v0);
            x.y = fmaf(a * b1, x.y, kd * v1);
            x.z = fmaf(a * b2, x.z, kd * v2);
            x.w = fmaf(a * b3, x.w, kd * v3);
            p[static_cast<size_t>(r) * ROWF4] = x;
            acc.x = fmaf(qw, x.x, acc.x);
            acc.y = fmaf(qw, x.y, acc.y);
            acc.z = fmaf(qw, x.z, acc.z);
            acc.w = fmaf(qw, x.w, acc.w);
        }
#pragma unroll
        for (int j = 0; j < ROWS; ++j) cur[j] = nxt[j];
    }

#pragma unroll
    for (int off = 32; off >= COLG; off >>= 1) {
        acc.x += __shfl_xor(acc.x, off);
        acc.y += __shfl_xor(acc.y, off);
        acc.z += __shfl_xor(acc.z, off);
        acc.w += __shfl_xor(acc.w, off);
    }
    const int wave = tid / 64, lane = tid % 64;
    if (lane < COLG) s_red[wave][lane] = acc;
    __syncthreads();
    if (tid < COLG) {
        float4 r = s_red[0][tid];
#pragma unroll
        for (int w = 1; w < kDecodeThreads / 64; ++w) {
            const float4 t = s_red[w][tid];
            r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w;
        }
        TIO *op = o + (trow * H + h) * DV + (part * COLG + tid) * 4;
        op[0] = from_f32<TIO>(r.x);
        op[1] = from_f32<TIO>(r.y);
        op[2] = from_f32<TIO>(r.z);
        op[3] = from_f32<TIO>(r.w);
    }
}

__global__ __launch_bounds__(256) void state_init_kernel(float4 *__restrict__ S1, float4 *__restrict__ S2, size_t n4)
{
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n4;
         i += static_cast<size_t>(gridDim.x) * blockDim.x) {
        S1[i] = z;
        S2[i] = z;
    }
}

// Two workgroups per (batch, head), each one half of the columns: measured fastest on MI355X (5.07 TB/s against
// 4.80 with one workgroup and 4.91 with four; non-temporal hints make no difference).
constexpr int kDecodeSplit = 2;

template <int D, class TIO, class TG>
hipError_t launch_decode_t(const dsla_desc &d, const void *q, const void *k, const void *v, const void *g1,
                           const void *g2, const int32_t *row, const int32_t *slot, float *S1, float *S2, void *o,
                           hipStream_t stream)
{
    const unsigned grid = static_cast<unsigned>(d.B) * static_cast<unsigned>(d.H) * kDecodeSplit;
    ProfileScope ps(DSLA_KERNEL_DECODE, stream);
    DSLA_LAUNCH(ps, (decode_kernel<D, D, kDecodeSplit, TIO, TG>), dim3(grid), dim3(kDecodeThreads), 0, stream,
                       static_cast<const TIO *>(q), static_cast<const TIO *>(k), static_cast<const TIO *>(v),
                       static_cast<const TG *>(g1), static_cast<const TG *>(g2), row, slot, S1, S2, static_cast<TIO *>(o), d.H,
                       d.gamma, d.gamma_per_head, d.scale, d.gate_mode == DSLA_GATE_PREACT ? 1.0f / d.tau : 0.f);
    return hipGetLastError();
}

template <int D>
hipError_t launch_decode_d(const dsla_desc &d, const void *q, const void *k, const void *v, const void *g1,
                           const void *g2, const int32_t *row, const int32_t *slot, float *S1, float *S2, void *o,
                           hipStream_t stream)
{
    const bool io16 = d.io_dtype == DSLA_BF16, g16 = d.gate_dtype == DSLA_BF16;
    if (io16 && g16) return launch_decode_t<D, bf16_t, bf16_t>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
    if (io16 && !g16) return launch_decode_t<D, bf16_t, float>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
    if (!io16 && g16) return launch_decode_t<D, float, bf16_t>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
    return launch_decode_t<D, float, float>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
}

template <int D, class TIO, class TG>
hipError_t launch_decode_multi_t(const dsla_desc &d, const MultiStatePtrs &mp, int N, int Hkv, const float *w_per_head,
                                 const void *q, const void *k, const void *v, const int32_t *row, const int32_t *slot,
                                 void *o, hipStream_t stream)
{
    const unsigned grid = static_cast<unsigned>(d.B) * static_cast<unsigned>(d.H) * kDecodeSplit;
    ProfileScope ps(DSLA_KERNEL_DECODE_MULTI, stream);
    DSLA_LAUNCH(ps, (decode_multi_kernel<D, D, kDecodeSplit, TIO, TG>), dim3(grid), dim3(kDecodeThreads), 0, stream,
                       static_cast<const TIO *>(q), static_cast<const TIO *>(k), static_cast<const TIO *>(v), mp, N, row, slot,
                       static_cast<TIO *>(o), d.H, Hkv, w_per_head, d.scale,
                       d.gate_mode == DSLA_GATE_PREACT ? 1.0f / d.tau : 0.f);
    return hipGetLastError();
}

template <int D>
hipError_t launch_decode_multi_d(const dsla_desc &d, const MultiStatePtrs &mp, int N, int Hkv, const float *w_per_head,
                                 const void *q, const void *k, const void *v, const int32_t *row, const int32_t *slot,
                                 void *o, hipStream_t stream)
{
    const bool io16 = d.io_dtype == DSLA_BF16, g16 = d.gate_dtype == DSLA_BF16;
    if (io16 && g16) return launch_decode_multi_t<D, bf16_t, bf16_t>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
    if (io16 && !g16) return launch_decode_multi_t<D, bf16_t, float>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
    if (!io16 && g16) return launch_decode_multi_t<D, float, bf16_t>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
    return launch_decode_multi_t<D, float, float>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
}

}  // namespace

hipError_t launch_decode_multi(const dsla_desc &d, const MultiStatePtrs &mp, int N, int Hkv, const float *w_per_head,
                               const void *q, const void *k, const void *v, const int32_t *row, const int32_t *slot,
                               void *o, hipStream_t stream)
{
    if (d.d_k == 128) return launch_decode_multi_d<128>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
    return launch_decode_multi_d<64>(d, mp, N, Hkv, w_per_head, q, k, v, row, slot, o, stream);
}

bool decode_supported(const dsla_desc &d) { return d.d_k == d.d_v && (d.d_k == 64 || d.d_k == 128); }

hipError_t launch_decode(const dsla_desc &d, const void *q, const void *k, const void *v, const void *g1,
                         const void *g2, const int32_t *row, const int32_t *slot, float *S1, float *S2, void *o,
                           hipStream_t stream)
{
    if (d.d_k == 128) return launch_decode_d<128>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
    return launch_decode_d<64>(d, q, k, v, g1, g2, row, slot, S1, S2, o, stream);
}

hipError_t launch_state_init(float *S1, float *S2, size_t elems_per_state, hipStream_t stream)
{
    const size_t n4 = elems_per_state / 4;  // d_k*d_v is a multiple of 4 for every supported shape
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks == 0) blocks = 1;
    ProfileScope ps(DSLA_KERNEL_STATE_INIT, stream);
    DSLA_LAUNCH(ps, state_init_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                       reinterpret_cast<float4 *>(S1), reinterpret_cast<float4 *>(S2), n4);
    return hipGetLastError();
}

}  // namespace dsla
