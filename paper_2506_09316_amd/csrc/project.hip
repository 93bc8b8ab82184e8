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
// (128 bytes per clock and CU) out of the way.  K in stages of 32 through a ring of four LDS stages (4 x 32 KB),
// filled by buffer loads that write LDS directly (no staging registers, no LDS store instructions): a load has two
// stages to arrive.  A row of a stage is 64 bytes, its four 16-byte pieces stored at piece position c ^ ((row / 4) % 4),
// so that the fragment reads of 16 lanes at a time touch every bank once.
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
constexpr int BM = 256, BN = 256;
constexpr int BK = 32;                            // values of K per stage
constexpr int ROWB = BK * 2;                     // bytes per LDS row: 64
constexpr int OPB = BM * ROWB;                  // bytes per operand tile and stage: 16 KB
constexpr int STAGEB = 2 * OPB;                 // A tile, then B tile: 32 KB

__global__ __launch_bounds__(256) void project_kernel_256(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                                 const float *__restrict__ bias, ProjectOuts outs, long long M,
                                                                 int K, int N, int width, int tiles_m, int tiles_n)
{
    // four stages as four objects: the compiler's wait-count insertion then knows that a load into one stage does not
    // touch what is read from another
    __shared__ __attribute__((aligned(1024))) char st0[STAGEB];
    __shared__ __attribute__((aligned(1024))) char st1[STAGEB];
    __shared__ __attribute__((aligned(1024))) char st2[STAGEB];
    __shared__ __attribute__((aligned(1024))) char st3[STAGEB];
    int tm, tn;
    if (!tile_of(tiles_m, tiles_n, tm, tn)) return;
    const long long m0 = static_cast<long long>(tm) * BM;
    const int n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;   // this wavefront's 128 x 128 quadrant
    const uint32_t uwave = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(wave));

    // Buffer loads with LDS as destination: one instruction of a wavefront fills 1 KB = 16 rows of 64 bytes of a
    // tile; instruction n = wave + 4 i (i < 4) fills rows 16 n .. 16 n + 15.  A lane fills LDS slot (row lane / 4, piece
    // position lane % 4) and fetches the piece that belongs there: piece c of row r sits at position c ^ ((r / 4) % 4),
    // so the 16 rows that 16 lanes read at the same logical piece fall into 16 different groups of four banks.  The
    // descriptor of an operand starts at the tile's first row and ends with the last row that exists: rows past the
    // end of x or W arrive as zeros.
    const long long rows_a = M - m0 < BM ? M - m0 : BM, rows_b = N - n0 < BN ? N - n0 : BN;
    const __amdgpu_buffer_rsrc_t res_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(x + static_cast<size_t>(m0) * K), 0, static_cast<int>(rows_a * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t res_b = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(w + static_cast<size_t>(n0) * K), 0, static_cast<int>(rows_b * K * 2), 0x00020000);
    uint32_t voff[4];   // byte offset of this lane's piece from the first row of the tile (the range check is on it)
#pragma unroll
    for (int i = 0; i < 4; ++i)
        voff[i] = (16 * (uwave + 4 * i) + (static_cast<uint32_t>(lane) >> 2)) * static_cast<uint32_t>(K) * 2u +
                  16 * ((lane & 3u) ^ ((static_cast<uint32_t>(lane) >> 4) & 3u));
    const int nk = K / BK;
    typedef __attribute__((address_space(3))) void *lds_void;
    auto fetch = [&](char *st, int ks) {   // K-step ks (past the end: the last one again, never used) into a stage
        const int kbyte = (ks < nk ? ks : nk - 1) * BK * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t n = uwave + 4 * i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(res_a, (lds_void)(st + n * 1024), 16, voff[i], kbyte, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(res_b, (lds_void)(st + OPB + n * 1024), 16, voff[i], kbyte, 0, 0);
        }
    };

    // fragment reads: row (quadrant + 32 i + ln) of a tile, block kb of 16 values of K: piece 2 kb + g
    const uint32_t swz = (ln >> 2) & 3;
    const uint32_t fo0 = ((0 + g) ^ swz) << 4, fo1 = ((2 + g) ^ swz) << 4;
    const uint32_t fa_row = static_cast<uint32_t>((128 * wm + ln) * ROWB);
    const uint32_t fb_row = static_cast<uint32_t>(OPB + (128 * wn + ln) * ROWB);
    bf16x8 fa[2][4], fb[2][4];   // fragments of two blocks: one in use, one arriving
    auto read_frags = [&](int buf, const char *st, int kb) {
        const uint32_t fo = kb ? fo1 : fo0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[buf][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(st + fa_row + i * 32 * ROWB + fo));
            fb[buf][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(st + fb_row + i * 32 * ROWB + fo));
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto block = [&](int kb) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kb][j], fa[kb][i], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                              // 1 MFMA
            if (t % 2 == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              // 1 LDS read
            if (kb == 0 && t % 2 == 1) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);   // 1 load into LDS
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // One K-step from stage `cur`.  On entry the fragments of its first block are in registers and stage `nxt` holds
    // what this wavefront loaded of the next step but one barrier short of being complete for everybody: the barrier
    // at the start certifies `nxt` (every wavefront has waited for its own loads of it: all but the 8 youngest, which
    // belong to the stage after) and frees `old` (everybody is done with the step before), which then takes K-step
    // ks + 3.  So a load has two steps to arrive, and no MFMA waits behind a barrier for LDS latency: the first
    // fragments of `nxt` are read during the second block.
    auto step = [&](const char *cur, const char *nxt, char *old, int ks) {
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        fetch(old, ks + 3);
        read_frags(1, cur, 1);
        block(0);
        read_frags(0, nxt, 0);
        block(1);
    };
    // nk is a multiple of 4 (K is a multiple of 128): the loop body has no branch, so the accumulators stay where they are
    fetch(st0, 0);
    fetch(st1, 1);
    fetch(st2, 2);
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");   // stage 0 is complete
    read_frags(0, st0, 0);
    __builtin_amdgcn_sched_barrier(0);
    for (int ks = 0; ks < nk; ks += 4) {
        step(st0, st1, st3, ks);
        step(st1, st2, st0, ks + 1);
        step(st2, st3, st1, ks + 2);
        step(st3, st0, st2, ks + 3);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // nothing in flight; everybody is done reading

    // Results: each wavefront turns its quadrant round in LDS - its own stage object, 128 rows of 256 bytes, the 16-byte
    // piece c of row r at position c ^ (r % 16) - so that it leaves as whole rows: a lane holds 4 adjacent columns of a
    // row per register group and writes them as 8 bytes; then 16 lanes read one row as 16 bytes each and store 256
    // contiguous bytes.
    char *epi = wave == 0 ? st0 : (wave == 1 ? st1 : (wave == 2 ? st2 : st3));
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
                const int row = 32 * i + ln, piece = cq >> 3;
                *reinterpret_cast<u32x2 *>(epi + row * 256 + ((piece ^ (row & 15)) << 4) + (cq & 4) * 2) = u32x2{pack2(c0, c1), pack2(c2, c3)};
            }
    if (nq < N) {
        bf16_t *out = static_cast<bf16_t *>(outs.p[nq / width]) + nq % width;
        const int rsub = lane >> 4, piece = lane & 15;   // 4 rows per instruction, 16 lanes per row
#pragma unroll 4
        for (int it = 0; it < 32; ++it) {
            const int row = 4 * it + rsub;
            const long long m = m0 + 128 * wm + row;
            const u32x4 vrow = *reinterpret_cast<const u32x4 *>(epi + row * 256 + ((piece ^ (row & 15)) << 4));
            if (m < M)   // streaming store: a tile of results is not read again by this kernel
                __builtin_nontemporal_store(vrow, reinterpret_cast<u32x4 *>(out + static_cast<size_t>(m) * width + piece * 8));
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
    if (K % (4 * BK) == 0) {   // the loop of project_kernel_256 goes four stages at a time
        const int tiles_m = static_cast<int>((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
        const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
        const unsigned grid = static_cast<unsigned>((ntiles + 7) / 8 * 8);
        DSLA_LAUNCH(ps, project_kernel_256, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(w), bias, po, static_cast<long long>(M), K, N, width, tiles_m, tiles_n);
    } else {
        const int tiles_m = static_cast<int>((M + TM - 1) / TM), tiles_n = N / TN;
        const long long ntiles = static_cast<long long>(tiles_m) * tiles_n;
        const unsigned grid = static_cast<unsigned>((ntiles + 7) / 8 * 8);
        DSLA_LAUNCH(ps, project_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(x),
                           static_cast<const bf16_t *>(w), bias, po, static_cast<long long>(M), K, width, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace dsla
