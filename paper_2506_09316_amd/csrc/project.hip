// The projections in front of a DSLA layer as one MFMA GEMM (paper Section 5.3: "single linear layers for gating";
// appendix on training details: the q, k, v projections are the teacher's own, the history gate's weight starts near
// the identity, the recency gate's from a normal distribution, biases zero): from the layer input x [M][K]
// (M = batch * tokens, K = model width) and the stacked weights W [n_out * width][K] it writes n_out tensors
// [M][width] - q, k, v and the two gate pre-activations - each laid out [B][T][H][d] as the prefill reads them, so
// nothing is permuted or converted in between; with gate_mode = DSLA_GATE_PREACT the prefill applies the gate map.
//     out_j[m][c] = sum_k x[m][k] W[j * width + c][k] (+ bias[j * width + c])
//
// Workgroup = 256 threads = 4 wavefronts on a 128 x 128 output tile (2 x 2 wavefronts, each 64 x 64 = four 32 x 32
// MFMA tiles), K in steps of 32 through double-buffered LDS; the next K-step's global loads are in flight while the
// current one is multiplied.  bf16 operands, fp32 accumulation, bf16 results.
#include "dsla_internal.h"

namespace dsla {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int PITCH = TK + 8;   // elements per LDS row: 80 bytes, conflict-free for the 16-byte fragment reads

struct ProjectOuts {
    void *p[DSLA_MAX_PROJECTIONS];
};

__device__ __forceinline__ uint32_t pack2(float a, float b)
{
    f32x2 x = {a, b};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return __builtin_bit_cast(uint32_t, y);
}

__global__ __launch_bounds__(256) void project_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                      const float *__restrict__ bias, ProjectOuts outs, long long M, int K,
                                                      int width, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][TM * PITCH];
    __shared__ __attribute__((aligned(16))) bf16_t sB[2][TN * PITCH];

    // Tile order: the 8 XCDs each take a contiguous run of the linear tile order (workgroup ids go round-robin over
    // the XCDs), inside which the row tile runs fastest: the 128 x K panel of W of a column tile stays in that XCD's
    // L2 while the rows stream past.
    const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
    const long long per_xcd = (ntiles + 7) / 8;
    const long long lin = static_cast<long long>(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (lin >= ntiles) return;
    const int tn = static_cast<int>(lin / tiles_m), tm = static_cast<int>(lin % tiles_m);
    const long long m0 = static_cast<long long>(tm) * TM;
    const int n0 = tn * TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;   // this wavefront's 64 x 64 quadrant

    // staging: 512 16-byte pieces per operand tile and K-step, two per thread: piece -> (row, 8 k-values)
    u32x4 ra[2], rb[2];
    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int piece = tid + 256 * i, row = piece >> 2, c = piece & 3;
            const long long m = m0 + row;
            ra[i] = u32x4{0, 0, 0, 0};
            if (m < M) ra[i] = *reinterpret_cast<const u32x4 *>(x + static_cast<size_t>(m) * K + k0 + 8 * c);
            rb[i] = *reinterpret_cast<const u32x4 *>(w + static_cast<size_t>(n0 + row) * K + k0 + 8 * c);
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int piece = tid + 256 * i, row = piece >> 2, c = piece & 3;
            *reinterpret_cast<u32x4 *>(&sA[buf][row * PITCH + 8 * c]) = ra[i];
            *reinterpret_cast<u32x4 *>(&sB[buf][row * PITCH + 8 * c]) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = K / TK;
    load_tiles(0);
    store_tiles(0);
    for (int ks = 0; ks < nk; ++ks) {
        __syncthreads();   // K-step ks is in buffer ks & 1; every wavefront is done with step ks - 1
        if (ks + 1 < nk) load_tiles((ks + 1) * TK);
        const bf16_t *a = sA[ks & 1], *b = sB[ks & 1];
        // acc[i][j] holds C^T tiles: result tile rows = output columns (from W), tile columns = output rows (from x),
        // so that a lane ends up with 4 adjacent output columns of one output row: 8-byte stores
#pragma unroll
        for (int kb = 0; kb < TK / 16; ++kb) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&a[(64 * wm + 32 * i + ln) * PITCH + 16 * kb + 8 * g]));
                fb[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&b[(64 * wn + 32 * i + ln) * PITCH + 16 * kb + 8 * g]));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (ks + 1 < nk) store_tiles((ks + 1) & 1);
    }

    // acc[i][j][r]: output row m0 + 64 wm + 32 i + ln, output column n0 + 64 wn + 32 j + 8 (r / 4) + 4 g + r % 4
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const long long m = m0 + 64 * wm + 32 * i + ln;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int rb4 = 0; rb4 < 4; ++rb4) {
                const int col = n0 + 64 * wn + 32 * j + 8 * rb4 + 4 * g;   // 4 adjacent columns, inside one output tensor
                float c0 = acc[i][j][4 * rb4], c1 = acc[i][j][4 * rb4 + 1], c2 = acc[i][j][4 * rb4 + 2], c3 = acc[i][j][4 * rb4 + 3];
                if (bias) {
                    c0 += bias[col];
                    c1 += bias[col + 1];
                    c2 += bias[col + 2];
                    c3 += bias[col + 3];
                }
                bf16_t *dst = static_cast<bf16_t *>(outs.p[col / width]) + static_cast<size_t>(m) * width + col % width;
                *reinterpret_cast<u32x2 *>(dst) = u32x2{pack2(c0, c1), pack2(c2, c3)};
            }
    }
}

}  // namespace

hipError_t launch_project(int64_t M, int K, int n_out, int width, const void *x, const void *w, const float *bias,
                          void *const *outs, hipStream_t stream)
{
    ProjectOuts po;
    for (int j = 0; j < DSLA_MAX_PROJECTIONS; ++j) po.p[j] = j < n_out ? outs[j] : nullptr;
    const int tiles_m = static_cast<int>((M + TM - 1) / TM), tiles_n = n_out * width / TN;
    const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
    const unsigned grid = static_cast<unsigned>((ntiles + 7) / 8 * 8);
    ProfileScope ps(DSLA_KERNEL_PROJECT, stream);
    hipLaunchKernelGGL(project_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                       static_cast<const bf16_t *>(w), bias, po, static_cast<long long>(M), K, width, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace dsla
