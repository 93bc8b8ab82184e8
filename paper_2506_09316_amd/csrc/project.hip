// The projections in front of a DSLA layer as one MFMA GEMM (paper Section 5.3: "single linear layers for gating";
// appendix on training details: the q, k, v projections are the teacher's own, the history gate's weight starts near
// the identity, the recency gate's from a normal distribution, biases zero): from the layer input x [M][K]
// (M = batch * tokens, K = model width) and the stacked weights W [n_out * width][K] it writes n_out tensors
// [M][width] - q, k, v and the two gate pre-activations - each laid out [B][T][H][d] as the prefill reads them, so
// nothing is permuted or converted in between; with gate_mode = DSLA_GATE_PREACT the prefill applies the gate map.
//     out_j[m][c] = sum_k x[m][k] W[j * width + c][k] (+ bias[j * width + c])
// bf16 operands, fp32 accumulation, bf16 results.  Two kernels:
//
// project_kernel_256 (K a multiple of 128): workgroup = 256 threads = 4 wavefronts on a 256 x 256 output tile, one
// wavefront per SIMD with a 128 x 128 quadrant = sixteen 32 x 32 MFMA tiles whose 256 accumulator registers live in
// the accumulation half of the register file.  Per 16 values of K a wavefront reads 4 + 4 fragments from LDS for 16
// MFMAs - half a 16-byte LDS read per MFMA, a quarter of what a 64 x 64 quadrant needs, which is what keeps the LDS
// (128 bytes per clock and CU) out of the way.  K in steps of 64 through double-buffered LDS (2 x 64 KB); a row of a
// tile is 128 bytes, its eight 16-byte pieces stored at piece position c ^ ((row / 2) % 8), so that both the staging
// stores and the fragment reads of 16 lanes at a time touch every bank once.
//
// project_kernel (any K that is a multiple of 32): 128 x 128 tile, 64 x 64 quadrants, K in steps of 32.
//
// Tile order, both kernels: see tile_of().
#include "dsla_internal.h"

#include <type_traits>

namespace dsla {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

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

// Tile order: the 8 XCDs each take a contiguous run of the linear tile order (workgroup ids go round-robin over the
// XCDs, each XCD has its own L2), and the linear order runs in groups of GM row tiles: inside a group the row tile
// runs fastest, then the column tile, so the tiles in flight at one time (a few dozen per XCD) share GM panels of x
// and a handful of panels of W instead of one panel of W and dozens of x.  False: no tile for this workgroup.
__device__ __forceinline__ bool tile_of(int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int GM = 8;
    const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
    const long long per_xcd = (ntiles + 7) / 8;
    const long long lin = static_cast<long long>(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (lin >= ntiles) return false;
    const long long per_group = static_cast<long long>(GM) * tiles_n;
    const int first_m = static_cast<int>(lin / per_group) * GM;
    const int gsz = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    const int in_group = static_cast<int>(lin % per_group);
    tn = in_group / gsz;
    tm = first_m + in_group % gsz;
    return true;
}

// One 32 x 32 result tile, held transposed (tile rows = output columns): register r of lane (ln, g) is output row
// m_tile + ln, output column n_tile + 8 (r / 4) + 4 g + r % 4, so a lane stores 4 adjacent columns at a time.
__device__ __forceinline__ void store_tile(const f32x16 &acc, const ProjectOuts &outs, const float *__restrict__ bias,
                                           long long m, int n_tile, int g, int width, int N)
{
#pragma unroll
    for (int rb4 = 0; rb4 < 4; ++rb4) {
        const int col = n_tile + 8 * rb4 + 4 * g;   // 4 adjacent columns, inside one output tensor
        if (col >= N) continue;
        float c0 = acc[4 * rb4], c1 = acc[4 * rb4 + 1], c2 = acc[4 * rb4 + 2], c3 = acc[4 * rb4 + 3];
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

// ---------------------------------------------------------------------------------------------------------------
// 256 x 256 tiles
// ---------------------------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROWB = BK * 2;                      // bytes per LDS row (one row of a tile, BK values of K)
constexpr int OPB = BM * ROWB;                    // bytes per operand tile: 32 KB
constexpr int STAGEB = 2 * OPB;                   // A tile, then B tile
constexpr int EPI_PITCH = 128 * 2 + 16;           // bytes per row of a wavefront's 128 x 128 result in LDS (padded)
constexpr int EPI_BYTES = 4 * 128 * EPI_PITCH;    // four wavefronts

__global__ __launch_bounds__(256) void project_kernel_256(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                          const float *__restrict__ bias, ProjectOuts outs, long long M,
                                                          int K, int N, int width, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(16))) char lds[EPI_BYTES > 2 * STAGEB ? EPI_BYTES : 2 * STAGEB];
    int tm, tn;
    if (!tile_of(tiles_m, tiles_n, tm, tn)) return;
    const long long m0 = static_cast<long long>(tm) * BM;
    const int n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;   // this wavefront's 128 x 128 quadrant

    // staging: 2048 16-byte pieces per operand tile and K-step, eight per thread: piece tid + 256 u is
    // (row tid / 8 + 32 u, 8 values of K from 8 (tid % 8)).  Buffer loads: the descriptor of an operand starts at the
    // tile's first row and ends with the last row that exists, so rows past the end of x or W read as zero; the
    // per-lane offset is 32 bits and the K-step is the scalar offset.
    const int srow = tid >> 3, sc = tid & 7;
    uint32_t goff[8];   // byte offset from the first row of the tile: the same in x and W
#pragma unroll
    for (int u = 0; u < 8; ++u) goff[u] = (static_cast<uint32_t>(srow + 32 * u) * static_cast<uint32_t>(K) + 8 * sc) * 2u;
    const long long rows_a = M - m0 < BM ? M - m0 : BM, rows_b = N - n0 < BN ? N - n0 : BN;
    const __amdgpu_buffer_rsrc_t res_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(x + static_cast<size_t>(m0) * K), 0, static_cast<int>(rows_a * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t res_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(w + static_cast<size_t>(n0) * K), 0, static_cast<int>(rows_b * K * 2), 0x00020000);
    // LDS position of this thread's pieces: (row / 2) % 8 is the same for all eight
    const uint32_t st_off = static_cast<uint32_t>(srow * ROWB + ((sc ^ ((srow >> 1) & 7)) << 4));

    // Two register sets for the staging: K-step j travels through set j % 2.  Its loads are issued at the start of
    // step j - 2 and it is written to LDS stage j % 2 during step j - 1, so a load has one to two steps (2048 MFMA
    // cycles each) to arrive.
    u32x4 ra[2][8], rb[2][8];
    auto load_tiles = [&](auto set, int k0) {
        constexpr int s = decltype(set)::value;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            ra[s][u] = __builtin_amdgcn_raw_buffer_load_b128(res_a, goff[u], k0 * 2, 0);
            rb[s][u] = __builtin_amdgcn_raw_buffer_load_b128(res_b, goff[u], k0 * 2, 0);
        }
    };
    auto store_tiles = [&](auto set, int u0, int u1) {   // pieces u0 .. u1 - 1 of set s -> LDS stage s
        constexpr int s = decltype(set)::value;
        char *base = lds + s * STAGEB + st_off;
#pragma unroll
        for (int u = u0; u < u1; ++u) {
            *reinterpret_cast<u32x4 *>(base + u * 32 * ROWB) = ra[s][u];
            *reinterpret_cast<u32x4 *>(base + OPB + u * 32 * ROWB) = rb[s][u];
        }
    };

    // fragment reads: row (quadrant + 32 i + ln) of a tile, K block kb: piece 2 kb + g at position (2 kb + g) ^ swz
    const uint32_t swz = (ln >> 1) & 7;
    uint32_t fo[BK / 16];
#pragma unroll
    for (int kb = 0; kb < BK / 16; ++kb) fo[kb] = ((2 * kb + g) ^ swz) << 4;
    const uint32_t fa_row = static_cast<uint32_t>((128 * wm + ln) * ROWB);
    const uint32_t fb_row = static_cast<uint32_t>(OPB + (128 * wn + ln) * ROWB);

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = K / BK;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    bf16x8 fa[2][4], fb[2][4];   // fragments of two blocks of 16 values of K: one in use, one arriving
    auto read_frags = [&](int buf, const char *st, int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[buf][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(st + fa_row + i * 32 * ROWB + fo[kb]));
            fb[buf][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(st + fb_row + i * 32 * ROWB + fo[kb]));
        }
    };
    // One K-step from LDS stage p: four blocks of 16 values of K, each 16 MFMAs with the other work of the block
    // spread between them one instruction at a time (a burst of LDS reads holds up the MFMA issue of a lone wavefront:
    // 1.24 against 1.35 PFLOP/s in a loop of nothing else).  The instruction scheduler is held to the order written
    // here; left alone it moves every fragment read down to just in front of its use.
    //   block 0: fragments of block 1; first half of K-step ks + 1 from its registers to the other stage; the loads
    //            of K-step ks + 2 into the registers K-step ks came through
    //   block 1: fragments of block 2; second half of K-step ks + 1
    //   barrier: the other stage is complete
    //   block 2: fragments of block 3
    //   block 3: fragments of block 0 of K-step ks + 1, from the other stage
    //   barrier: everybody is done reading this stage; the next step may overwrite it
    // so no MFMA ever waits for a barrier and the LDS latency behind it.  On entry the fragments of block 0 are there.
    auto block = [&](int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kb & 1][j], fa[kb & 1][i], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                             // 1 MFMA
            // blocks in front of a barrier (1 and 3) have their LDS work in the first three quarters, so that it is
            // done when the wavefront arrives there
            if (kb % 2 == 0 ? t % 2 == 0 : t < 8) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
            if (kb == 0 ? t % 2 == 1 : (kb == 1 && t >= 4 && t < 12)) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // 1 LDS store
            if (kb == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                // 1 global load
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto step = [&](auto par, int ks) {
        constexpr int p = decltype(par)::value;
        using Other = std::integral_constant<int, 1 - p>;
        const char *st = lds + p * STAGEB, *sn = lds + (1 - p) * STAGEB;
        read_frags(1, st, 1);
        store_tiles(Other{}, 0, 4);   // after the last step: the last step again, into a stage nobody reads any more
        load_tiles(par, (ks + 2 < nk ? ks + 2 : nk - 1) * BK);   // past the end: the last step again, never used
        block(0);
        read_frags(0, st, 2);
        store_tiles(Other{}, 4, 8);
        block(1);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, st, 3);
        block(2);
        read_frags(0, sn, 0);
        block(3);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };
    // nk is even (K is a multiple of 2 BK): the loop body has no branch, so the accumulators stay where they are
    load_tiles(P0{}, 0);
    load_tiles(P1{}, BK);
    store_tiles(P0{}, 0, 8);
    __syncthreads();
    read_frags(0, lds, 0);
    __builtin_amdgcn_sched_barrier(0);
    for (int ks = 0; ks < nk; ks += 2) {
        step(P0{}, ks);
        step(P1{}, ks + 1);
    }

    // Results: each wavefront turns its quadrant round in LDS (its own 34 KB; the last barrier of the loop has freed the
    // stages) so that it leaves as whole rows: a lane holds 4 adjacent columns of a row per register group and writes
    // them as 8 bytes; then 16 lanes read one row of 128 columns as 16 bytes each and store 256 contiguous bytes.
    // (Stored straight from the registers, 8 bytes at a time into 32 different rows per instruction, the results of a
    // tile took an eighth of the kernel's time.)
    char *epi = lds + wave * (128 * EPI_PITCH);
    const int nq = n0 + 128 * wn;   // first column of the quadrant: inside one output tensor (width is a multiple of 128)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int rb4 = 0; rb4 < 4; ++rb4) {
                const int cq = 32 * j + 8 * rb4 + 4 * g;   // column inside the quadrant
                float c0 = acc[i][j][4 * rb4], c1 = acc[i][j][4 * rb4 + 1], c2 = acc[i][j][4 * rb4 + 2], c3 = acc[i][j][4 * rb4 + 3];
                if (bias && nq + cq < N) {
                    const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + nq + cq);
                    c0 += bv[0];
                    c1 += bv[1];
                    c2 += bv[2];
                    c3 += bv[3];
                }
                *reinterpret_cast<u32x2 *>(epi + (32 * i + ln) * EPI_PITCH + cq * 2) = u32x2{pack2(c0, c1), pack2(c2, c3)};
            }
    if (nq < N) {
        bf16_t *out = static_cast<bf16_t *>(outs.p[nq / width]) + nq % width;
        const int rsub = lane >> 4, piece = lane & 15;   // 4 rows per instruction, 16 lanes per row
#pragma unroll 4
        for (int it = 0; it < 32; ++it) {
            const int row = 4 * it + rsub;
            const long long m = m0 + 128 * wm + row;
            const u32x4 vrow = *reinterpret_cast<const u32x4 *>(epi + row * EPI_PITCH + piece * 16);
            if (m < M) *reinterpret_cast<u32x4 *>(out + static_cast<size_t>(m) * width + piece * 8) = vrow;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// 128 x 128 tiles
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void project_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                      const float *__restrict__ bias, ProjectOuts outs, long long M, int K,
                                                      int width, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][TM * PITCH];
    __shared__ __attribute__((aligned(16))) bf16_t sB[2][TN * PITCH];

    int tm, tn;
    if (!tile_of(tiles_m, tiles_n, tm, tn)) return;
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

#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const long long m = m0 + 64 * wm + 32 * i + ln;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) store_tile(acc[i][j], outs, bias, m, n0 + 64 * wn + 32 * j, g, width, tiles_n * TN);
    }
}

}  // namespace

hipError_t launch_project(int64_t M, int K, int n_out, int width, const void *x, const void *w, const float *bias,
                          void *const *outs, hipStream_t stream)
{
    ProjectOuts po;
    for (int j = 0; j < DSLA_MAX_PROJECTIONS; ++j) po.p[j] = j < n_out ? outs[j] : nullptr;
    const int N = n_out * width;
    ProfileScope ps(DSLA_KERNEL_PROJECT, stream);
    if (K % (2 * BK) == 0) {
        const int tiles_m = static_cast<int>((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
        const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
        const unsigned grid = static_cast<unsigned>((ntiles + 7) / 8 * 8);
        hipLaunchKernelGGL(project_kernel_256, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(w), bias, po, static_cast<long long>(M), K, N, width, tiles_m, tiles_n);
    } else {
        const int tiles_m = static_cast<int>((M + TM - 1) / TM), tiles_n = N / TN;
        const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
        const unsigned grid = static_cast<unsigned>((ntiles + 7) / 8 * 8);
        hipLaunchKernelGGL(project_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(w), bias, po, static_cast<long long>(M), K, width, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace dsla
