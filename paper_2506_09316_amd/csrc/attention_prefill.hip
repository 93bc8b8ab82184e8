// Causal softmax attention over a whole prompt: the prefill of a layer that has NOT been converted, which a partly
// converted model runs beside its DSLA layers (paper Section 4.3) and against which the linear-time DSLA prefill is
// measured (Section 5.3: quadratic against linear cost, crossing near 2K tokens).
//     o_t = sum_{i <= t} softmax_{i <= t}(scale * q_t . k_i) v_i
//
// One pass over the keys with a running reference maximum (the scores never leave the chip).  A workgroup of four
// wavefronts takes 128 consecutive queries of one (batch, head); a wavefront owns 32 of them.  Keys and values stream
// through LDS 64 at a time, shared by the four wavefronts, by buffer loads that go from memory straight to LDS (no
// staging registers, no LDS store instructions; see AttnTiles for the placement that keeps the reads conflict-free).
// Per block of 64 keys a wavefront computes two transposed score tiles S^T[key][query] = K Q^T on MFMA (so that a lane
// holds the scores of ONE query: the softmax needs one cross-lane exchange), exponentiates against the reference, and
// adds V^T P^T to its output tiles O^T[column][query].
// The causal mask is applied only in the blocks on the diagonal, and the reference is raised (and the output tiles
// rescaled) only when a block exceeds it by more than 2^8, which after the first blocks is rare.  Because an MFMA
// result tile and an MFMA input fragment both index lanes by the tile column, the exponentiated tile is fed back as
// the input fragment of the second product without passing through LDS; V sits in LDS as its rows arrived and its
// transposed fragments come from the transposing LDS read, in the key order the result registers of a score tile have.
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

constexpr int kWaves = 4;                                 // wavefronts per workgroup
constexpr int kQueriesPerWg = 32 * kWaves;
constexpr int kKeys = 64;            // keys per block: two score tiles of 32
// The running maximum of a query is only raised when a block exceeds it by more than this (log2 units): the
// exponentials then stay below 2^8 and the output tiles are rescaled once in a long while instead of once per block.
// The normalisation at the end uses the same reference for numerator and denominator, so the result is the same sum.
constexpr float kMaxSlack = 8.0f;

__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    f32x2 x = {a, b};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return __builtin_bit_cast(uint32_t, y);
}
// LDS image of a block of 64 keys (and of its values): rows of d elements WITHOUT padding, because the block is
// written by loads that go from memory straight to LDS (a wavefront's 64 lanes fill 1 KB of consecutive LDS).  Bank
// conflicts are avoided by WHERE in its row a 16-byte piece is put:
// - keys: piece c of row r sits at piece position c ^ swz_k(r); the 16 rows that 16 lanes read at one time at the
//   same logical piece then fall into 16 different groups of four banks;
// - values: the 64-byte quarter q of row r sits at quarter position q ^ swz_v(r); a pass of the transposing read
//   takes one quarter from each of 4 consecutive rows, which then fall into the four quarters of the banks.
// The lane that fills LDS slot (row, position) simply fetches the piece that belongs there.
template <int D>
struct AttnTiles {
    static constexpr int RB = D * 2;                    // bytes per row
    static constexpr int NC = D / 8;                    // 16-byte pieces per row (16 or 8)
    static constexpr int NQ = RB / 64;                  // 64-byte quarters per row (4 or 2)
    static constexpr uint32_t K_BYTES = kKeys * RB;
    static constexpr uint32_t V_BYTES = kKeys * RB;
    static constexpr uint32_t BUF_BYTES = K_BYTES + V_BYTES;
    static __device__ __forceinline__ uint32_t swz_k(uint32_t row) { return NC == 16 ? (row & 15u) : ((row >> 1) & 7u); }
    static __device__ __forceinline__ uint32_t swz_v(uint32_t row) { return NQ == 4 ? (row & 3u) : ((row >> 1) & 1u); }
};

// Fragment of V^T for a block of 16 keys from V rows in LDS, by two transposing 8-byte reads: the 16 lanes of a group
// address 4 keys x 4 pieces of 4 columns and each receives 4 keys of ONE column.  With `a` as computed in the kernel
// lane l ends up with column (tile) + l % 32 and keys 4 g + 0..3 (from a) and 8 + 4 g + 0..3 (from a + 8 rows): the
// order in which the result registers of a score tile hold the keys.
__device__ __forceinline__ bf16x8 load_vt_frag(const char *a, uint32_t eight_rows)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef s16x4 __attribute__((address_space(3))) *lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a + eight_rows));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    return __builtin_bit_cast(bf16x8, u32x4{l2[0], l2[1], h2[0], h2[1]});
}

template <int D>
__global__ __launch_bounds__(64 * kWaves, 512 / (64 * kWaves)) void attention_prefill_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                                   const bf16_t *__restrict__ v, bf16_t *__restrict__ o,
                                                                   int H, int T, int blocks_per_seq, float scale_log2e)
{
    using L = AttnTiles<D>;
    constexpr int NKB = D / 16;    // contraction blocks over the features
    constexpr int CT = D / 32;     // output column tiles
    // two buffers as two objects: the compiler then knows that a load into one does not touch what is read from the other
    __shared__ __attribute__((aligned(1024))) char buf_a[L::BUF_BYTES];
    __shared__ __attribute__((aligned(1024))) char buf_b[L::BUF_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    // heavy blocks (late queries: more keys) first
    const int bh = blockIdx.x / blocks_per_seq;
    const int qb = blocks_per_seq - 1 - blockIdx.x % blocks_per_seq;
    const int b = bh / H, h = bh % H;
    const int q0 = qb * kQueriesPerWg;
    const size_t rs = static_cast<size_t>(H) * D;                                   // elements between tokens
    const size_t base = (static_cast<size_t>(b) * T * H + h) * D;                   // (b, 0, h, 0)

    // ---- this lane's query: features 16 kb + 8 g .. + 7 for every kb, scaled by scale * log2 e, as bf16 ----
    const int wq0 = q0 + 32 * wave;   // first query of this wavefront
    const int my_q = wq0 + ln;
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

    // ---- staging of a key/value block: buffer loads with LDS as destination.  One instruction of a wavefront fills
    // 1 KB = RPI rows; instruction n = wave + kWaves i of a block fills rows n RPI .. of the keys (and one more of the
    // values).  The descriptors cover this (batch, head)'s keys and values from token 0 to the end of the last token's
    // row: rows past the end of the sequence arrive as zeros (they lie after every query and are masked). ----
    constexpr int RPI = 1024 / L::RB;                  // rows per instruction (4 or 8)
    constexpr int NI = kKeys / RPI / kWaves;           // instructions per wavefront, block and tensor
    static_assert(NI >= 1, "every wavefront stages something");
    const uint32_t rs2 = static_cast<uint32_t>(rs) * 2;   // bytes between tokens
    const int kv_bytes = static_cast<int>(static_cast<uint32_t>(T - 1) * rs2 + D * 2);   // an unsigned 32-bit count to the hardware
    const __amdgpu_buffer_rsrc_t res_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(k + base), 0, kv_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t res_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(v + base), 0, kv_bytes, 0x00020000);
    const uint32_t uwave = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(wave));
    // this lane's LDS slot in an instruction: row lr of its RPI rows, piece position lp; the swizzles of the rows an
    // instruction fills depend on the lane and the wavefront only (RPI n is a multiple of what they look at)
    const uint32_t lr = static_cast<uint32_t>(lane) / L::NC, lp = static_cast<uint32_t>(lane) % L::NC;
    const uint32_t row0 = RPI * uwave + lr;            // row of instruction i = 0
    const uint32_t goff_k = lr * rs2 + 16 * (lp ^ L::swz_k(row0));
    const uint32_t goff_v = lr * rs2 + 16 * ((((lp >> 2) ^ L::swz_v(row0)) << 2) | (lp & 3u));
    auto stage_block = [&](char *buf, int key0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t n = uwave + kWaves * i;
            // the range check is on the lane offset alone, so the row goes into it
            const uint32_t rowoff = (static_cast<uint32_t>(key0) + RPI * n) * rs2;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(res_k, (__attribute__((address_space(3))) void *)(buf + n * 1024), 16,
                                                     rowoff + goff_k, 0, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(res_v, (__attribute__((address_space(3))) void *)(buf + L::K_BYTES + n * 1024), 16,
                                                     rowoff + goff_v, 0, 0, 0);
        }
    };
    // fragment reads.  Keys: row 32 t + ln, logical piece 2 kb + g.  Values (transposing reads): the 16 lanes of a
    // group address 4 rows x 4 pieces of 4 columns: row 4 g + l16 / 4 of a block of 16 keys (+ 8 for the second read),
    // columns 32 ct + 16 (lane / 16 % 2) + 4 (l16 % 4), i.e. quarter ct of the row.
    const uint32_t sk = L::swz_k(ln);                  // (rows 32 t + ln: the swizzle looks at the low bits only)
    const uint32_t kf_off = ln * L::RB + 16 * ((g ^ sk) & 1u);
    const uint32_t kf_s1 = sk >> 1;                    // piece pair kb of the row sits at pair position kb ^ kf_s1
    const uint32_t l16 = lane & 15;
    const uint32_t vrow = 4 * g + (l16 >> 2);
    const uint32_t sv = L::swz_v(vrow);                // (rows 16 kb2 + 8 h + vrow: low bits only)
    const uint32_t vt_off = vrow * L::RB + 32 * ((lane >> 4) & 1) + 8 * (l16 & 3);

    // keys this workgroup needs: 0 .. min(T, q0 + 128) - 1; this wavefront needs them up to its last query
    const int wg_last_q = (q0 + kQueriesPerWg < T ? q0 + kQueriesPerWg : T) - 1;
    const int nblocks = wg_last_q / kKeys + 1;
    const int wave_last_q = wq0 + 31;

    f32x16 oacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[ct][r] = 0.f;
    float m_ref = -1.0e30f, l_run = 0.f;   // reference maximum (log2 domain) and denominator of this lane's query

    auto compute = [&](const char *buf, int jb) {
        const int key0 = jb * kKeys;
        if (key0 <= wave_last_q) {   // else: every key of the block lies after every query of this wavefront
            const char *kb_ = buf;
            const char *vb_ = buf + L::K_BYTES;
            // S^T[key][query], two tiles of 32 keys: lane (ln, g) ends up with keys 32 t + 8 (r / 4) + 4 g + r % 4 of query ln
            f32x16 sc[2];
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(kb_ + 32 * t * L::RB + kf_off + 32 * (kb ^ kf_s1)));
                    sc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kb], kb ? sc[t] : zero, 0, 0, 0);
                }
            // causal mask, only in the blocks that reach past the first query of the wavefront (keys past the end of
            // the sequence lie after every query)
            if (key0 + kKeys - 1 > wq0) {
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
                        sc[t][r] = key <= my_q ? sc[t][r] : -1.0e30f;
                    }
            }
            float bmax = fmaxf(sc[0][0], sc[1][0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) bmax = fmaxf(bmax, fmaxf(sc[0][r], sc[1][r]));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            // raise the reference of every query when any query of the wavefront needs it (uniform branch)
            if (__builtin_amdgcn_ballot_w64(bmax > m_ref + kMaxSlack) != 0) {
                const float m_new = fmaxf(m_ref, bmax);
                const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
                l_run *= alpha;
                m_ref = m_new;
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[ct][r] *= alpha;
            }
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    sc[t][r] = __builtin_amdgcn_exp2f(sc[t][r] - m_ref);   // masked entries: 2^(-1e30 - m) = 0
                    psum += sc[t][r];
                }
            psum += __shfl_xor(psum, 32);
            l_run += psum;
            // the halves of the tiles as the input fragments of the four blocks of 16 keys
            bf16x8 pf[4];
#pragma unroll
            for (int kb2 = 0; kb2 < 4; ++kb2) {
                const f32x16 &x = sc[kb2 >> 1];
                const int o8 = 8 * (kb2 & 1);
                const u32x4 u = {pack2(x[o8 + 0], x[o8 + 1]), pack2(x[o8 + 2], x[o8 + 3]), pack2(x[o8 + 4], x[o8 + 5]),
                                 pack2(x[o8 + 6], x[o8 + 7])};
                pf[kb2] = __builtin_bit_cast(bf16x8, u);
            }
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int kb2 = 0; kb2 < 4; ++kb2) {
                    const bf16x8 vf = load_vt_frag(vb_ + vt_off + 16 * kb2 * L::RB + 64 * (ct ^ sv), 8 * L::RB);
                    oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb2], oacc[ct], 0, 0, 0);
                }
        }
    };
    // Block j lives in buffer j % 2; its loads are issued one iteration ahead, right after the barrier that frees the
    // buffer, and the barrier in front of its use waits for them (the loads of every wavefront must have landed).
    stage_block(buf_a, 0);
    for (int jb = 0; jb < nblocks; jb += 2) {
        __syncthreads();   // block jb is in buffer a; every wavefront is done with block jb - 1
        if (jb + 1 < nblocks) stage_block(buf_b, (jb + 1) * kKeys);
        compute(buf_a, jb);
        if (jb + 1 < nblocks) {
            __syncthreads();   // block jb + 1 is in buffer b; every wavefront is done with block jb
            if (jb + 2 < nblocks) stage_block(buf_a, (jb + 2) * kKeys);
            compute(buf_b, jb + 1);
        }
    }

    // ---- o[query][32 ct + 8 (r / 4) + 4 g + r % 4] = O^T / denominator ----
    if (q_live) {
        const float inv = 1.0f / l_run;   // the query's own key is never masked: l_run > 0
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
        DSLA_LAUNCH(ps, (attention_prefill_kernel<128>), dim3(grid), dim3(64 * kWaves), 0, stream, static_cast<const bf16_t *>(q),
                           static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), H,
                           static_cast<int>(T), blocks_per_seq, sl2);
    else
        DSLA_LAUNCH(ps, (attention_prefill_kernel<64>), dim3(grid), dim3(64 * kWaves), 0, stream, static_cast<const bf16_t *>(q),
                           static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), H,
                           static_cast<int>(T), blocks_per_seq, sl2);
    return hipGetLastError();
}

}  // namespace dsla
