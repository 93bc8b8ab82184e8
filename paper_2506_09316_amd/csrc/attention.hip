// The two softmax-attention pieces that stand beside the DSLA layer in the paper's serving system, both for ONE
// query per (batch, head) against T keys, both bandwidth-bound single passes over [B][T][H][d] tensors:
//
//  * attention entropy of the final query (Section 4.3, "Layer Ranking via Sensitivity"): the softmax distribution
//    of scale * q_T . k_i over the keys and its Shannon entropy H = -sum_i A_i log A_i, the signal the paper ranks
//    layers by before converting them;
//  * single-query attention over a key/value cache: the decode step of a layer that has not been converted,
//    o = sum_i A_i v_i, whose cost grows with the context while the DSLA decode step's does not (Section 5.3).
//
// One pass with a running maximum.  A group of lanes that together hold one key row keeps
//     m = max s,   z = sum e^(s - m),   and   w = sum e^(s - m) (s - m)   or   acc = sum e^(s - m) v
// (H = log z - w / z, o = acc / z).  Two such records merge exactly (up to rounding), so the keys of one
// (batch, head) can be split over several workgroups when there are too few pairs to fill the chip; a second small
// kernel merges the parts.  Keys and values are read once, as whole rows, with the non-temporal hint.
#include "dsla_internal.h"

namespace dsla {
namespace {

constexpr int kEntThreads = 256;
constexpr int kEntUnroll = 8;   // key rows in flight per lane group

struct Part {
    float m, z, w;
};
// "no keys yet": z = 0 and a finite, very small maximum, so that no infinity enters the arithmetic
__device__ __forceinline__ Part empty_part() { return Part{-1.0e30f, 0.f, 0.f}; }
__device__ __forceinline__ void rebase(Part &a, float m_new)
{
    const float c = expf(a.m - m_new);
    a.w = c * (a.w + a.z * (a.m - m_new));
    a.z = c * a.z;
    a.m = m_new;
}
__device__ __forceinline__ void merge(Part &a, Part b)
{
    const float m = fmaxf(a.m, b.m);
    rebase(a, m);
    rebase(b, m);
    a.z += b.z;
    a.w += b.w;
}

// The keys are read once and whole rows at a time: the non-temporal hint is worth 10-15 % of bandwidth here.
__device__ __forceinline__ void load8(const bf16_t *p, float (&f)[8])
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f[2 * w] = __uint_as_float(u[w] << 16);
        f[2 * w + 1] = __uint_as_float(u[w] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8(const float *p, float (&f)[8])
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 4));
    f[0] = a[0]; f[1] = a[1]; f[2] = a[2]; f[3] = a[3];
    f[4] = b[0]; f[5] = b[1]; f[6] = b[2]; f[7] = b[3];
}

// A lane holds 8 adjacent features of a key row; LPR = D / 8 lanes hold a row; the workgroup's 256 lanes hold
// 256 / LPR rows at a time.  Workgroup (bh, part) takes the keys [part * rows_per_part, ...) of its (batch, head).
template <int D, class TIO>
__global__ __launch_bounds__(kEntThreads) void entropy_kernel(const TIO *__restrict__ q_last, const TIO *__restrict__ k,
                                                              float scale, int H, long long T, int P,
                                                              long long rows_per_part, float *__restrict__ parts,
                                                              float *__restrict__ entropy)
{
    constexpr int LPR = D / 8;
    constexpr int GROUPS = kEntThreads / LPR;
    __shared__ Part s_part[GROUPS];

    const int bh = blockIdx.x / P, part = blockIdx.x % P;
    const int b = bh / H, h = bh % H;
    const int grp = threadIdx.x / LPR, c = threadIdx.x % LPR;
    const long long t0 = part * rows_per_part;
    const long long t1 = (t0 + rows_per_part < T) ? t0 + rows_per_part : T;

    float qf[8];
    load8(q_last + (static_cast<size_t>(bh) * D + 8 * c), qf);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] *= scale;

    const size_t pitch = static_cast<size_t>(H) * D;   // elements between consecutive keys
    const TIO *kb = k + (static_cast<size_t>(b) * T * H + h) * D + 8 * c;
    Part acc = empty_part();
    for (long long t = t0 + grp; t < t1; t += static_cast<long long>(GROUPS) * kEntUnroll) {
        float kf[kEntUnroll][8];
#pragma unroll
        for (int u = 0; u < kEntUnroll; ++u) {   // rows past the end re-read the last row and are masked below
            long long row = t + static_cast<long long>(u) * GROUPS;
            row = row < t1 ? row : t1 - 1;
            load8(kb + static_cast<size_t>(row) * pitch, kf[u]);
        }
        float s[kEntUnroll];
        float mb = -1.0e30f;
#pragma unroll
        for (int u = 0; u < kEntUnroll; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qf[e], kf[u][e], d);
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
            const bool valid = t + static_cast<long long>(u) * GROUPS < t1;
            s[u] = valid ? d : -1.0e30f;
            mb = fmaxf(mb, s[u]);
        }
        if (mb > acc.m) rebase(acc, mb);   // uniform within the lane group
#pragma unroll
        for (int u = 0; u < kEntUnroll; ++u) {
            const float x = s[u] - acc.m;          // <= 0; a masked row gives e^(-huge) = 0
            const float e = __expf(x);
            acc.z += e;
            acc.w = fmaf(e, fmaxf(x, -1.0e4f), acc.w);   // (the clamp keeps 0 * huge out of the sum)
        }
    }
    if (c == 0) s_part[grp] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        Part r = s_part[0];
        for (int g = 1; g < GROUPS; ++g) merge(r, s_part[g]);
        if (P == 1) {
            entropy[bh] = logf(r.z) - r.w / r.z;
        } else {
            float *o = parts + (static_cast<size_t>(bh) * P + part) * 3;
            o[0] = r.m;
            o[1] = r.z;
            o[2] = r.w;
        }
    }
}

__global__ __launch_bounds__(256) void entropy_merge_kernel(const float *__restrict__ parts, int BH, int P,
                                                            float *__restrict__ entropy)
{
    const int bh = blockIdx.x * blockDim.x + threadIdx.x;
    if (bh >= BH) return;
    const float *p = parts + static_cast<size_t>(bh) * P * 3;
    Part r{p[0], p[1], p[2]};
    for (int i = 1; i < P; ++i) merge(r, Part{p[3 * i], p[3 * i + 1], p[3 * i + 2]});
    entropy[bh] = logf(r.z) - r.w / r.z;
}

// ---- single-query attention over cached keys and values -------------------------------------------------------
template <class TIO>
struct RawRow;   // the 8 elements of a row a lane holds, as loaded
template <>
struct RawRow<bf16_t> {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 u;
    __device__ __forceinline__ void load(const bf16_t *p) { u = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)); }
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
struct RawRow<float> {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    f32x4 a, b;
    __device__ __forceinline__ void load(const float *p)
    {
        a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        b = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 4));
    }
    __device__ __forceinline__ void unpack(float (&f)[8]) const
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            f[w] = a[w];
            f[4 + w] = b[w];
        }
    }
};

// Same decomposition as entropy_kernel; a part's record is (m, z, acc[D]).
template <int D, class TIO>
__global__ __launch_bounds__(kEntThreads) void attn_decode_kernel(const TIO *__restrict__ q_last, const TIO *__restrict__ k,
                                                                  const TIO *__restrict__ v,
                                                                  const int32_t *__restrict__ seq_lens, float scale,
                                                                  int H, long long T, int P, long long rows_per_part,
                                                                  float *__restrict__ parts, TIO *__restrict__ o)
{
    constexpr int LPR = D / 8;
    constexpr int GROUPS = kEntThreads / LPR;
    constexpr int UNR = sizeof(TIO) == 2 ? 8 : 4;   // key/value row pairs in flight per lane group
    __shared__ float s_m[GROUPS], s_z[GROUPS];
    __shared__ float s_acc[GROUPS][D];

    const int bh = blockIdx.x / P, part = blockIdx.x % P;
    const int b = bh / H, h = bh % H;
    const int grp = threadIdx.x / LPR, c = threadIdx.x % LPR;
    // the cache of sequence b holds Tb <= T positions (its rows stay T apart); a part past the end leaves an empty record
    const long long Tb = seq_lens ? static_cast<long long>(seq_lens[b]) : T;
    const long long t0 = part * rows_per_part;
    const long long t1 = (t0 + rows_per_part < Tb) ? t0 + rows_per_part : Tb;

    float qf[8];
    load8(q_last + (static_cast<size_t>(bh) * D + 8 * c), qf);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] *= scale;

    const size_t pitch = static_cast<size_t>(H) * D;
    const size_t base = (static_cast<size_t>(b) * T * H + h) * D + 8 * c;
    float m = -1.0e30f, z = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    for (long long t = t0 + grp; t < t1; t += static_cast<long long>(GROUPS) * UNR) {
        RawRow<TIO> kr[UNR], vr[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {   // rows past the end re-read the last row and are masked below
            long long row = t + static_cast<long long>(u) * GROUPS;
            row = row < t1 ? row : t1 - 1;
            kr[u].load(k + base + static_cast<size_t>(row) * pitch);
            vr[u].load(v + base + static_cast<size_t>(row) * pitch);
        }
        float s[UNR];
        float mb = -1.0e30f;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float kf[8];
            kr[u].unpack(kf);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qf[e], kf[e], d);
#pragma unroll
            for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
            const bool valid = t + static_cast<long long>(u) * GROUPS < t1;
            s[u] = valid ? d : -1.0e30f;
            mb = fmaxf(mb, s[u]);
        }
        if (mb > m) {   // uniform within the lane group
            const float c0 = expf(m - mb);
            z *= c0;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= c0;
            m = mb;
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const float w = __expf(s[u] - m);   // a masked row: e^(-huge) = 0
            float vf[8];
            vr[u].unpack(vf);
            z += w;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, vf[e], acc[e]);
        }
    }
    if (c == 0) {
        s_m[grp] = m;
        s_z[grp] = z;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[grp][8 * c + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {   // thread f merges feature f over the lane groups
        const int f = threadIdx.x;
        float M = s_m[0];
        for (int g = 1; g < GROUPS; ++g) M = fmaxf(M, s_m[g]);
        float Z = 0.f, A = 0.f;
        for (int g = 0; g < GROUPS; ++g) {
            const float c0 = expf(s_m[g] - M);
            Z = fmaf(c0, s_z[g], Z);
            A = fmaf(c0, s_acc[g][f], A);
        }
        if (P == 1) {
            o[static_cast<size_t>(bh) * D + f] = from_f32<TIO>(A / Z);
        } else {
            float *rec = parts + (static_cast<size_t>(bh) * P + part) * (2 + D);
            if (f == 0) {
                rec[0] = M;
                rec[1] = Z;
            }
            rec[2 + f] = A;
        }
    }
}

template <int D, class TIO>
__global__ __launch_bounds__(D) void attn_decode_merge_kernel(const float *__restrict__ parts, int P, TIO *__restrict__ o)
{
    const int bh = blockIdx.x, f = threadIdx.x;
    const float *rec = parts + static_cast<size_t>(bh) * P * (2 + D);
    float M = rec[0];
    for (int i = 1; i < P; ++i) M = fmaxf(M, rec[static_cast<size_t>(i) * (2 + D)]);
    float Z = 0.f, A = 0.f;
    for (int i = 0; i < P; ++i) {
        const float *r = rec + static_cast<size_t>(i) * (2 + D);
        const float c0 = expf(r[0] - M);
        Z = fmaf(c0, r[1], Z);
        A = fmaf(c0, r[2 + f], A);
    }
    o[static_cast<size_t>(bh) * D + f] = from_f32<TIO>(A / Z);
}

template <int D, class TIO>
hipError_t launch_attn_decode_t(int B, int H, int64_t T, const EntropyPlan &plan, float scale, const void *q_last,
                                const void *k, const void *v, const int32_t *seq_lens, void *o, void *workspace,
                                hipStream_t stream)
{
    const int BH = B * H;
    ProfileScope ps(DSLA_KERNEL_ATTENTION_DECODE, stream);
    if (plan.parts == 1) ps.e1_first = ps.e1;   // no merge kernel follows: the first launch closes the record too
    DSLA_LAUNCH_FIRST(ps, (attn_decode_kernel<D, TIO>), dim3(static_cast<unsigned>(BH) * plan.parts), dim3(kEntThreads), 0,
                       stream, static_cast<const TIO *>(q_last), static_cast<const TIO *>(k), static_cast<const TIO *>(v),
                       seq_lens, scale, H, static_cast<long long>(T), plan.parts, static_cast<long long>(plan.rows_per_part),
                       static_cast<float *>(workspace), static_cast<TIO *>(o));
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || plan.parts == 1) return err;
    DSLA_LAUNCH_LAST(ps, (attn_decode_merge_kernel<D, TIO>), dim3(BH), dim3(D), 0, stream,
                       static_cast<const float *>(workspace), plan.parts, static_cast<TIO *>(o));
    return hipGetLastError();
}

template <int D, class TIO>
hipError_t launch_entropy_t(int B, int H, int64_t T, const EntropyPlan &plan, float scale, const void *q_last,
                            const void *k, float *entropy, void *workspace, hipStream_t stream)
{
    const int BH = B * H;
    ProfileScope ps(DSLA_KERNEL_ATTENTION_ENTROPY, stream);
    if (plan.parts == 1) ps.e1_first = ps.e1;   // no merge kernel follows: the first launch closes the record too
    DSLA_LAUNCH_FIRST(ps, (entropy_kernel<D, TIO>), dim3(static_cast<unsigned>(BH) * plan.parts), dim3(kEntThreads), 0, stream,
                       static_cast<const TIO *>(q_last), static_cast<const TIO *>(k), scale, H, static_cast<long long>(T),
                       plan.parts, static_cast<long long>(plan.rows_per_part), static_cast<float *>(workspace), entropy);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || plan.parts == 1) return err;
    DSLA_LAUNCH_LAST(ps, entropy_merge_kernel, dim3((BH + 255) / 256), dim3(256), 0, stream,
                       static_cast<const float *>(workspace), BH, plan.parts, entropy);
    return hipGetLastError();
}

}  // namespace

bool entropy_plan(int B, int H, int d, int64_t T, EntropyPlan *plan, int floats_per_part)
{
    if (d != 64 && d != 128) return false;
    const int64_t BH = static_cast<int64_t>(B) * H;
    // two workgroups per compute unit (measured at 8 x 32 pairs of 8192 keys: 90 us; one: 102 us; four: 97 us),
    // at least 256 keys per workgroup
    int64_t P = (512 + BH - 1) / BH;
    const int64_t most = (T + 255) / 256;
    if (P > most) P = most;
    if (P < 1) P = 1;
    plan->rows_per_part = (T + P - 1) / P;
    plan->parts = static_cast<int>((T + plan->rows_per_part - 1) / plan->rows_per_part);
    plan->ws_bytes = plan->parts > 1 ? static_cast<size_t>(BH) * plan->parts * floats_per_part * sizeof(float) : 0;
    return true;
}

hipError_t launch_entropy(int B, int H, int d, int64_t T, int io_dtype, const EntropyPlan &plan, float scale,
                          const void *q_last, const void *k, float *entropy, void *workspace, hipStream_t stream)
{
    if (io_dtype == DSLA_BF16) {
        if (d == 128) return launch_entropy_t<128, bf16_t>(B, H, T, plan, scale, q_last, k, entropy, workspace, stream);
        if (d == 64) return launch_entropy_t<64, bf16_t>(B, H, T, plan, scale, q_last, k, entropy, workspace, stream);
    } else {
        if (d == 128) return launch_entropy_t<128, float>(B, H, T, plan, scale, q_last, k, entropy, workspace, stream);
        if (d == 64) return launch_entropy_t<64, float>(B, H, T, plan, scale, q_last, k, entropy, workspace, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_attn_decode(int B, int H, int d, int64_t T, int io_dtype, const EntropyPlan &plan, float scale,
                              const void *q_last, const void *k, const void *v, const int32_t *seq_lens, void *o,
                              void *workspace, hipStream_t stream)
{
    if (io_dtype == DSLA_BF16) {
        if (d == 128) return launch_attn_decode_t<128, bf16_t>(B, H, T, plan, scale, q_last, k, v, seq_lens, o, workspace, stream);
        if (d == 64) return launch_attn_decode_t<64, bf16_t>(B, H, T, plan, scale, q_last, k, v, seq_lens, o, workspace, stream);
    } else {
        if (d == 128) return launch_attn_decode_t<128, float>(B, H, T, plan, scale, q_last, k, v, seq_lens, o, workspace, stream);
        if (d == 64) return launch_attn_decode_t<64, float>(B, H, T, plan, scale, q_last, k, v, seq_lens, o, workspace, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace dsla
