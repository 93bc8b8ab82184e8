// Causal softmax attention over a whole prompt: the prefill of a layer that has NOT been converted, which a partly
// converted model runs beside its DSLA layers (paper Section 4.3) and against which the linear-time DSLA prefill is
// measured (Section 5.3: quadratic against linear cost, crossing near 2K tokens).
//     o_t = sum_{i <= t} softmax_{i <= t}(scale * q_t . k_i) v_i
//
// One pass over the keys with a running maximum (the scores never leave the chip).  A workgroup of four wavefronts
// takes 128 consecutive queries of one (batch, head); a wavefront owns 32 of them.  Keys and values stream through
// LDS 32 at a time, shared by the four wavefronts.  Per block of 32 keys a wavefront computes the transposed score
// tile S^T[key][query] = K Q^T on MFMA (so that a lane holds the scores of ONE query: the softmax needs one
// cross-lane exchange), exponentiates against the running maximum, and adds V^T P^T to its output tiles
// O^T[column][query].  Because an MFMA result tile and an MFMA input fragment both index lanes by the tile column, the
// exponentiated tile is fed back as the input fragment of the second product without passing through LDS; V is
// stored in LDS with the matching order of the keys (bits 2 and 3 of the key index swapped).
// bf16 operands, fp32 accumulation and softmax statistics.
#include "dsla_internal.h"

namespace dsla {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kQueriesPerWg = 128;   // 4 wavefronts x 32
constexpr int kKeys = 32;            // keys per block

__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    f32x2 x = {a, b};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return __builtin_bit_cast(uint32_t, y);
}
// bits 2 and 3 of an index swapped: with the keys of V stored in this order, the 8 result registers of half a 32x32
// tile (lane group g holds tile rows 8a + 4g + b) are the 8 contraction indices lane group g supplies as an input.
__device__ __forceinline__ uint32_t rho(uint32_t x) { return (x & ~12u) | ((x & 4u) << 1) | ((x & 8u) >> 1); }

template <int D>
struct AttnTiles {
    static constexpr int KP = D + 8;                              // pitch of a key row (elements): conflict-free 16-byte reads
    static constexpr uint32_t K_BYTES = kKeys * KP * 2;
    static constexpr uint32_t V_BYTES = D * kKeys * 2;            // [column][32 keys], piece c of row R at c ^ ((R / 2) % 4)
    static constexpr uint32_t BUF_BYTES = K_BYTES + V_BYTES;
};

template <int D>
__global__ __launch_bounds__(256) void attention_prefill_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                                const bf16_t *__restrict__ v, bf16_t *__restrict__ o,
                                                                int H, long long T, int blocks_per_seq, float scale_log2e)
{
    using L = AttnTiles<D>;
    constexpr int NKB = D / 16;    // contraction blocks over the features
    constexpr int CT = D / 32;     // output column tiles
    __shared__ __attribute__((aligned(16))) char smem[2 * L::BUF_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    // heavy blocks (late queries: more keys) first
    const int bh = blockIdx.x / blocks_per_seq;
    const int qb = blocks_per_seq - 1 - blockIdx.x % blocks_per_seq;
    const int b = bh / H, h = bh % H;
    const long long q0 = static_cast<long long>(qb) * kQueriesPerWg;
    const size_t rs = static_cast<size_t>(H) * D;                                   // elements between tokens
    const size_t base = (static_cast<size_t>(b) * T * H + h) * D;                   // (b, 0, h, 0)

    // ---- this lane's query: features 16 kb + 8 g .. + 7 for every kb, scaled by scale * log2 e, as bf16 ----
    const long long my_q = q0 + 32 * wave + ln;
    const bool q_live = my_q < T;
    bf16x8 qf[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        u32x4 u = {0, 0, 0, 0};
        if (q_live) u = *reinterpret_cast<const u32x4 *>(q + base + static_cast<size_t>(my_q) * rs + 16 * kb + 8 * g);
        u32x4 s;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            s[w] = pack2(__uint_as_float(u[w] << 16) * scale_log2e, __uint_as_float(u[w] & 0xffff0000u) * scale_log2e);
        qf[kb] = __builtin_bit_cast(bf16x8, s);
    }

    // ---- staging of a key/value block: thread -> (key row, 16-byte pieces) and (key pair, 8 columns) ----
    constexpr int KPIECES = kKeys * D / 8 / 256;   // 16-byte pieces of K per thread (2 at D = 128, 1 at D = 64)
    constexpr int VTHREADS = 16 * D / 8;           // threads that stage V (a pair of keys x 8 columns each)
    const int vpair = tid / (D / 8), vcol = 8 * (tid % (D / 8));
    u32x4 kreg[KPIECES], vreg[2];
    auto load_block = [&](long long key0) {
#pragma unroll
        for (int i = 0; i < KPIECES; ++i) {
            const int piece = tid + 256 * i, row = piece / (D / 8), c = piece % (D / 8);
            const long long key = key0 + row;
            kreg[i] = u32x4{0, 0, 0, 0};
            if (key < T) kreg[i] = *reinterpret_cast<const u32x4 *>(k + base + static_cast<size_t>(key) * rs + 8 * c);
        }
        if (tid < VTHREADS) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const long long key = key0 + 2 * vpair + j;
                vreg[j] = u32x4{0, 0, 0, 0};
                if (key < T) vreg[j] = *reinterpret_cast<const u32x4 *>(v + base + static_cast<size_t>(key) * rs + vcol);
            }
        }
    };
    auto store_block = [&](int buf) {
        char *kb_ = smem + buf * L::BUF_BYTES;
        char *vb_ = kb_ + L::K_BYTES;
#pragma unroll
        for (int i = 0; i < KPIECES; ++i) {
            const int piece = tid + 256 * i, row = piece / (D / 8), c = piece % (D / 8);
            *reinterpret_cast<u32x4 *>(kb_ + (row * L::KP + 8 * c) * 2) = kreg[i];
        }
        if (tid < VTHREADS) {
            const uint32_t tok = rho(2 * vpair), tpiece = tok >> 3, within = tok & 7;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                const uint32_t two = __builtin_amdgcn_perm(vreg[1][e >> 1], vreg[0][e >> 1], sel);   // (key 2p, key 2p+1) of column e
                const uint32_t row = vcol + e;
                *reinterpret_cast<uint32_t *>(vb_ + (row * kKeys + 8 * (tpiece ^ ((row >> 1) & 3u)) + within) * 2) = two;
            }
        }
    };

    // keys this workgroup needs: 0 .. min(T, q0 + 128) - 1; this wavefront needs them up to its last query
    const long long wg_last_q = (q0 + kQueriesPerWg < T ? q0 + kQueriesPerWg : T) - 1;
    const int nblocks = static_cast<int>(wg_last_q / kKeys) + 1;
    const long long wave_last_q = q0 + 32 * wave + 31;

    f32x16 oacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[ct][r] = 0.f;
    float m_run = -1.0e30f, l_run = 0.f;   // running maximum (log2 domain) and denominator of this lane's query

    load_block(0);
    store_block(0);
    for (int jb = 0; jb < nblocks; ++jb) {
        __syncthreads();   // block jb is in buffer jb & 1; every wavefront is done with block jb - 1
        if (jb + 1 < nblocks) load_block(static_cast<long long>(jb + 1) * kKeys);
        const long long key0 = static_cast<long long>(jb) * kKeys;
        if (key0 <= wave_last_q) {   // else: every key of the block lies after every query of this wavefront
            const char *kb_ = smem + (jb & 1) * L::BUF_BYTES;
            const char *vb_ = kb_ + L::K_BYTES;
            // S^T[key][query]: lane (ln, g) ends up with keys 8 (r / 4) + 4 g + r % 4 of query ln
            f32x16 sc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(kb_ + (ln * L::KP + 16 * kb + 8 * g) * 2));
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kb], sc, 0, 0, 0);
            }
            // causal mask and keys past the end
            float bmax = -1.0e30f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long key = key0 + 8 * (r >> 2) + 4 * g + (r & 3);
                sc[r] = (key <= my_q && key < T) ? sc[r] : -1.0e30f;
                bmax = fmaxf(bmax, sc[r]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            const float m_new = fmaxf(m_run, bmax);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sc[r] = __builtin_amdgcn_exp2f(sc[r] - m_new);   // masked entries: 2^(-1e30 - m) = 0
                psum += sc[r];
            }
            psum += __shfl_xor(psum, 32);
            l_run = l_run * alpha + psum;
            m_run = m_new;
            // the two halves of the tile as the input fragments of the two blocks of 16 keys
            bf16x8 pf[2];
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {
                const u32x4 u = {pack2(sc[8 * kb2 + 0], sc[8 * kb2 + 1]), pack2(sc[8 * kb2 + 2], sc[8 * kb2 + 3]),
                                 pack2(sc[8 * kb2 + 4], sc[8 * kb2 + 5]), pack2(sc[8 * kb2 + 6], sc[8 * kb2 + 7])};
                pf[kb2] = __builtin_bit_cast(bf16x8, u);
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[ct][r] *= alpha;
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2) {
                    const uint32_t row = 32 * ct + ln;
                    const uint32_t piece = (g + 2 * kb2) ^ ((row >> 1) & 3u);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(vb_ + (row * kKeys + 8 * piece) * 2));
                    oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb2], oacc[ct], 0, 0, 0);
                }
            }
        }
        if (jb + 1 < nblocks) store_block((jb + 1) & 1);
    }

    // ---- o[query][32 ct + 8 (r / 4) + 4 g + r % 4] = O^T / denominator ----
    if (q_live) {
        const float inv = 1.0f / l_run;   // the query's own key is never masked: l_run >= 1
        bf16_t *op = o + base + static_cast<size_t>(my_q) * rs;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
                *reinterpret_cast<u32x2 *>(op + 32 * ct + 8 * rb + 4 * g) =
                    u32x2{pack2(oacc[ct][4 * rb] * inv, oacc[ct][4 * rb + 1] * inv),
                          pack2(oacc[ct][4 * rb + 2] * inv, oacc[ct][4 * rb + 3] * inv)};
    }
}

}  // namespace

hipError_t launch_attn_prefill(int B, int H, int d, int64_t T, float scale, const void *q, const void *k, const void *v,
                               void *o, hipStream_t stream)
{
    const int blocks_per_seq = static_cast<int>((T + kQueriesPerWg - 1) / kQueriesPerWg);
    const unsigned grid = static_cast<unsigned>(B) * H * blocks_per_seq;
    const float sl2 = scale * 1.4426950408889634f;
    ProfileScope ps(DSLA_KERNEL_ATTENTION_PREFILL, stream);
    if (d == 128)
        hipLaunchKernelGGL((attention_prefill_kernel<128>), dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(q),
                           static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), H,
                           static_cast<long long>(T), blocks_per_seq, sl2);
    else
        hipLaunchKernelGGL((attention_prefill_kernel<64>), dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(q),
                           static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), H,
                           static_cast<long long>(T), blocks_per_seq, sl2);
    return hipGetLastError();
}

}  // namespace dsla
