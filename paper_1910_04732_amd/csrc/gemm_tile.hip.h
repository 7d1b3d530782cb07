// Grouped MFMA tile kernel for the contractions of the gated factorized layer.
//
// One launch executes up to eight independent products C = op(A) op(B) whose
// output tiles are laid end to end in the grid, so that small products (the
// shapes of Section 4.1 are a few GFLOP each) still fill 256 compute units.
// Each operand is described by its own layout flag, which covers the three
// shapes the layer needs with row-major storage:
//     forward      x Q^T, g P^T        A[m,k] and B[n,k]   (k contiguous, k contiguous)
//     dg, dx       dy P,  dh Q         A[m,k] and B[k,n]   (k contiguous, n contiguous)
//     dP, dQ       dy^T g, dh^T x      A[k,m] and B[k,n]   (m contiguous, n contiguous)
// Tiles are staged through LDS in a [row][k] layout (rows padded by 16 bytes so
// that 16-byte fragment reads are bank-conflict free); operands whose
// contiguous dimension is not k are transposed in registers on the way in.
// Products are accumulated in float32 by v_mfma_f32_32x32x16_bf16 (bfloat16) or
// v_mfma_f32_32x32x2_f32 (float32).  The epilogue can scale column n by a gate
// z[n] before the single rounding.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_kernels.hip.h"

namespace flop {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kGemmThreads = 256;
constexpr int kMaxGroup = 8;
constexpr int kTileBand = 8;   // tile rows per band of the tile numbering (see locate_tile)
constexpr int kStepBytes = 128;            // bytes of k staged per main-loop step
constexpr int kLdsRow = kStepBytes + 16;   // padded LDS row

struct GemmProblem {
    const void* A;
    const void* B;
    void* C;
    const float* col_scale;   // nullable: C[m,n] = acc[m,n] * col_scale[n]
    // Alternative to col_scale (asynchronous-transfer kernel only): the scale of column n is the train-mode
    // Hard-Concrete gate of (gate_alpha[n], gate_u[n]), computed in the epilogue (see gate_one).
    const float* gate_alpha;
    const float* gate_u;
    float gate_beta, gate_l, gate_r;
    int64_t lda, ldb, ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int xcd_begin;            // first per-XCD block index of this problem (see locate_tile)
    int tiles_per_xcd;        // ceil(tiles_m * tiles_n / 8)
    int a_kmajor;             // 1: A[m*lda + k]   0: A[k*lda + m]
    int b_kmajor;             // 1: B[n*ldb + k]   0: B[k*ldb + n]
    int a_vec, b_vec;         // 16-byte loads allowed (alignment of base and ld)
    // Optional extent known only on the device (token buckets of the embedding path):
    const int32_t* seg;       // nullable: {first row, row count}
    const int32_t* c_rowmap;  // nullable: row i of the product goes to row c_rowmap[first + i] of C
    int seg_dim;              // 1: the segment is the M extent, 2: the K extent (host M or K is its upper bound)
    int seg_a, seg_b, seg_c;  // whether the operand's rows along that extent start at `first row`
    // Optional extent read from one device int (the active rank after compaction): replaces
    // M (ext_dim 1), K (2) or N (3); the host value is its upper bound and sizes the grid.
    const int32_t* ext;
    int ext_dim;
    // Optional split of the k extent over ksplit blocks per tile (few tiles, long k): block
    // `slice` contracts k in [slice * chunk, (slice + 1) * chunk) and stores its float32
    // accumulators, unscaled, to split_out[slice][M][N]; splitk_reduce_kernel adds the slices.
    int ksplit;               // 0 or 1: no split
    float* split_out;
    // Optional column reduction fused into the epilogue (asynchronous-transfer kernel only):
    // dot_partial[tile_m * N + n] = sum over the tile's rows m of C[m,n] * dot[m,n], C as stored.
    const void* dot;          // nullable: M x N matrix of the element type, rows at least 4-byte aligned
    int64_t lddot;
    float* dot_partial;       // tiles_m rows of dot_ld floats
    int64_t dot_ld;           // the host's N (a device-side extent does not change the row pitch)
    // Optional gather of B by an index list (the open components of a layer, ascending): the product runs on the
    // rows b_map[0 .. extent) of the b_map_rows-row matrix at B - its rows n when b_kmajor (B[n][k] = matrix row
    // b_map[n]), its k rows otherwise (B[k][n] = matrix row b_map[k]).  No compacted copy of the matrix is needed.
    const int32_t* b_map;
    int b_map_rows;
};

struct GemmGroup {
    GemmProblem p[kMaxGroup];
    int count;
    // Optional rider (asynchronous-transfer kernel only): blocks tile_blocks .. tile_blocks + rider_blocks - 1 of
    // the launch do the step-boundary work instead of a tile.
    int tile_blocks, rider_blocks;
    BoundaryRider rider;
    // Alternative block -> tile mapping for launches of several products with host-known extents (see locate_tile):
    // the products' tiles form one sequence, product after product, and XCD x works on its tiles
    // xcd_first[x] .. xcd_first[x + 1] - 1; p[q].xcd_begin is then product q's first position in that sequence.
    int contiguous;
    int xcd_first[9];
#ifdef FLOP_PHASE_STAMPS
    int stamp_slot;   // measurement build: where this launch's blocks record their phase times, or -1
#endif
};

// Head of a launch: what a block of the launch's first product needs to start its main loop, passed as leading
// scalar kernel arguments.  The kernels are compiled with kernel-argument preloading, so these arrive in registers
// with the wavefront, while the group itself (by value, in the kernel-argument segment) is a trip to memory away:
// 1.4 us per block before the first transfer could be issued, measured with per-block timestamps, a quarter of a
// launch of 8 us.  The rest of the first product's descriptor (output, scales, column sums) is read from the
// group after the main loop.  Blocks of later products, and launches whose first product has device-side
// extents, a gathered operand or a k split, take everything from the group as before (flags == 0).
struct LaunchHead {
    const void* A;
    const void* B;
    uint32_t lda, ldb;
    int M, N, K;
    int flags;   // kHeadValid | kHeadAKmajor | kHeadBKmajor
    int next;    // per-XCD block indices below this belong to the first product (its tiles_per_xcd)
};
constexpr int kHeadValid = 1, kHeadAKmajor = 2, kHeadBKmajor = 4;
#define FLOP_HEAD_PARAMS const void* hA, const void* hB, uint32_t hlda, uint32_t hldb, int hM, int hN, int hK, int hflags, int hnext
#define FLOP_HEAD_ARGS LaunchHead{hA, hB, hlda, hldb, hM, hN, hK, hflags, hnext}

// Tiles are numbered band by band: a band is kTileBand tile rows, walked column by
// column, so that the tiles in flight on an XCD share few row and column panels.
template <int BM, int BN>
__device__ __forceinline__ void decode_tile(const GemmProblem& pr, int t, int& tile_m, int& tile_n)
{
    // a tile twice as tall as wide has row panels twice the size of its column panels: half as many tile rows per band
    // keep the bytes of the panels that the tiles in flight on an XCD share at their minimum
    constexpr int kTileBand = BM > BN ? flop::kTileBand / 2 : flop::kTileBand;
    const int band_tiles = kTileBand * pr.tiles_n;
    const int band = t / band_tiles, in_band = t - band * band_tiles;
    const int rows_here = min(kTileBand, pr.tiles_m - band * kTileBand);
    tile_n = in_band / rows_here;
    tile_m = band * kTileBand + (in_band - tile_n * rows_here);
}

// Block -> (problem, tile).  Hardware hands consecutive block ids to the eight
// XCDs in turn, each with its own L2.  Every problem's tile list is cut into
// eight contiguous ranges, one per XCD, so that an XCD re-uses operand panels
// in its own L2 and every XCD gets the same share of every problem (they differ
// in k extent).  Block b serves XCD b%8 with per-XCD index b/8; problems are
// laid out one after another along that index, each padded to tiles_per_xcd
// entries.  Returns false for padding blocks, which have no tile.
// from_head: the problem was built from the launch head; its epilogue fields are still to be read (finish_problem)
template <int ES, int BM, int BN>
__device__ __forceinline__ bool locate_tile(const LaunchHead& head, const GemmGroup& grp, GemmProblem& pr, int& tile_m,
                                            int& tile_n, bool& from_head)
{
    const int xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    from_head = (head.flags & kHeadValid) != 0 && i < head.next;
    if (from_head) {
        pr = GemmProblem{};
        pr.A = head.A; pr.B = head.B;
        pr.lda = head.lda; pr.ldb = head.ldb;
        pr.M = head.M; pr.N = head.N; pr.K = head.K;
        pr.tiles_m = (head.M + BM - 1) / BM;
        pr.tiles_n = (head.N + BN - 1) / BN;
        pr.tiles_per_xcd = head.next;
        pr.a_kmajor = (head.flags & kHeadAKmajor) != 0;
        pr.b_kmajor = (head.flags & kHeadBKmajor) != 0;
        const int t = xcd * head.next + i;
        if (t >= pr.tiles_m * pr.tiles_n) return false;
        decode_tile<BM, BN>(pr, t, tile_m, tile_n);
        return true;
    }
    if (grp.contiguous) {
        // One sequence of tiles cut into eight contiguous pieces of equal work: a product lies on as few XCDs as
        // its size allows, so that its operand panels are fetched into few L2s (weight-gradient products of many
        // layers in one launch: every operand is as long as the token count and used by one product only).
        const int pos = grp.xcd_first[xcd] + i;
        if (pos >= grp.xcd_first[xcd + 1]) return false;
        pr = grp.p[0];
        int q = 0;
#pragma unroll
        for (int j = 1; j < kMaxGroup; ++j) q += (j < grp.count && pos >= grp.p[j].xcd_begin) ? 1 : 0;
        if (q != 0) pr = grp.p[q];
        decode_tile<BM, BN>(pr, pos - pr.xcd_begin, tile_m, tile_n);
        return true;
    }
    // The group lies in the kernel-argument segment, a trip to memory away (0.8 us measured per dependent load at the
    // start of a block).  The first product's descriptor is fetched together with the products' starting
    // positions instead of after them: that is the only product of a forward launch and, products being ordered by
    // k extent, the one with the longest tiles of a grouped launch; only blocks of later products pay a second trip.
    pr = grp.p[0];
    int q = 0;   // xcd_begin ascends: the problem's index is the number of later problems that start at or before i
#pragma unroll
    for (int j = 1; j < kMaxGroup; ++j) q += (j < grp.count && i >= grp.p[j].xcd_begin) ? 1 : 0;
    if (q != 0) pr = grp.p[q];
    // Extents known only on the device shrink the problem first, so that the tiles that remain
    // are again spread evenly over the XCDs (the grid was sized for the host's upper bounds).
    if (pr.seg) {
        const int first = pr.seg[0], cnt = pr.seg[1];
        if (pr.seg_dim == 1) pr.M = cnt; else pr.K = cnt;
        if (pr.seg_a) pr.A = (const char*)pr.A + (int64_t)first * pr.lda * ES;
        if (pr.seg_b) pr.B = (const char*)pr.B + (int64_t)first * pr.ldb * ES;
        if (pr.seg_c) pr.C = (char*)pr.C + (int64_t)first * pr.ldc * ES;
        if (pr.c_rowmap) pr.c_rowmap += first;
    }
    if (pr.ext) {
        const int v = pr.ext[0];
        if (pr.ext_dim == 1) pr.M = min(pr.M, v);
        else if (pr.ext_dim == 2) pr.K = min(pr.K, v);
        else pr.N = min(pr.N, v);
    }
    const int slices = pr.ksplit > 1 ? pr.ksplit : 1;
    if (pr.seg || pr.ext) {
        pr.tiles_m = (pr.M + BM - 1) / BM;
        pr.tiles_n = (pr.N + BN - 1) / BN;
        pr.tiles_per_xcd = (pr.tiles_m * pr.tiles_n * slices + 7) / 8;
    }
    int t = xcd * pr.tiles_per_xcd + (i - pr.xcd_begin);
    if ((i - pr.xcd_begin) >= pr.tiles_per_xcd || t >= pr.tiles_m * pr.tiles_n * slices) return false;
    if (slices > 1) {
        // slices of one tile are far apart in the numbering: an XCD works on neighbouring tiles of one slice
        const int per_slice = pr.tiles_m * pr.tiles_n;
        const int slice = t / per_slice;
        t -= slice * per_slice;
        const int steps = (pr.K + 63) / 64;
        const int chunk = ((steps + slices - 1) / slices) * 64;
        const int k0 = slice * chunk;
        const int k_here = max(0, min(chunk, pr.K - k0));
        pr.A = (const char*)pr.A + (int64_t)k0 * (pr.a_kmajor ? 1 : pr.lda) * ES;
        pr.B = (const char*)pr.B + (int64_t)k0 * (pr.b_kmajor ? 1 : pr.ldb) * ES;
        pr.K = k_here;
        pr.split_out += (int64_t)slice * pr.M * pr.N;
    }
    decode_tile<BM, BN>(pr, t, tile_m, tile_n);
    return true;
}

// The fields of the first product that its blocks did not need before the main loop (see LaunchHead).
__device__ __forceinline__ void finish_problem(GemmProblem& pr, const GemmProblem& g)
{
    pr.C = g.C; pr.ldc = g.ldc;
    pr.col_scale = g.col_scale;
    pr.gate_alpha = g.gate_alpha; pr.gate_u = g.gate_u;
    pr.gate_beta = g.gate_beta; pr.gate_l = g.gate_l; pr.gate_r = g.gate_r;
    pr.c_rowmap = g.c_rowmap;
    pr.a_vec = g.a_vec; pr.b_vec = g.b_vec;
    pr.dot = g.dot; pr.lddot = g.lddot; pr.dot_partial = g.dot_partial; pr.dot_ld = g.dot_ld;
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b)
{
    return __builtin_bit_cast(float, b << 16);
}

// 16 bytes of `base[src_row*ld + col ...]` (src_row: where row lies in memory, row itself unless the operand is
// gathered), zero where row >= rows or col+e >= cols.
template <int ES>
__device__ __forceinline__ u32x4 load_vec16(const void* base, int64_t ld, int row, int col,
                                            int rows, int cols, bool vec_ok, int src_row)
{
    constexpr int E = 16 / ES;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (row < rows && col < cols) {
        const char* p = (const char*)base + ((int64_t)src_row * ld + col) * ES;
        if (vec_ok && col + E <= cols) {
            v = *(const u32x4*)p;
        } else if constexpr (ES == 2) {
            const uint16_t* q = (const uint16_t*)p;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                uint32_t x = (col + e < cols) ? (uint32_t)q[e] : 0u;
                v[e >> 1] |= x << (16 * (e & 1));
            }
        } else {
            const uint32_t* q = (const uint32_t*)p;
#pragma unroll
            for (int e = 0; e < E; ++e) v[e] = (col + e < cols) ? q[e] : 0u;
        }
    }
    return v;
}

// Global -> register -> LDS staging of one operand tile of ROWS rows by
// kStepBytes of k.  Each thread owns ROWS/32 sixteen-byte vectors.
template <int ES, int ROWS>
struct TileStager {
    static constexpr int NV = ROWS / 32;
    static constexpr int E = 16 / ES;
    static constexpr int BK = kStepBytes / ES;
    static constexpr int VPR = ROWS * ES / 16;   // vectors per k-row when rows are contiguous
    u32x4 v[NV];

    // map (nullable): the operand's rows (kmajor) or k rows (otherwise) are rows map[i] of the matrix at base
    __device__ __forceinline__ void load(const void* base, int64_t ld, int kmajor, bool vec_ok,
                                         int row0, int k0, int rows, int K, int tid, const int32_t* map = nullptr)
    {
        if (kmajor) {
            const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
            for (int p = 0; p < NV; ++p) {
                const int row = row0 + r0 + 32 * p;
                const int src = (map && row < rows) ? map[row] : row;
                v[p] = load_vec16<ES>(base, ld, row, k0 + c * E, rows, K, vec_ok, src);
            }
        } else {
            const int mv = tid % VPR, kq = tid / VPR;
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                const int k = k0 + kq * NV + q;
                const int src = (map && k < K) ? map[k] : k;
                v[q] = load_vec16<ES>(base, ld, k, row0 + mv * E, K, rows, vec_ok, src);
            }
        }
    }

    __device__ __forceinline__ void store(unsigned char* lds, int kmajor, int tid) const
    {
        if (kmajor) {
            const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
            for (int p = 0; p < NV; ++p)
                *(u32x4*)(lds + (r0 + 32 * p) * kLdsRow + c * 16) = v[p];
        } else {
            const int mv = tid % VPR, kq = tid / VPR;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                unsigned char* dst = lds + (mv * E + j) * kLdsRow + kq * NV * ES;
                if constexpr (ES == 2) {
                    // 16-bit element j of vector q; NV of them are packed in k order
                    auto el = [&](int q) { return (v[q][j >> 1] >> (16 * (j & 1))) & 0xFFFFu; };
                    if constexpr (NV == 1) {
                        *(uint16_t*)dst = (uint16_t)el(0);
                    } else if constexpr (NV == 2) {
                        *(uint32_t*)dst = el(0) | (el(1) << 16);
                    } else if constexpr (NV == 4) {
                        *(u32x2*)dst = u32x2{el(0) | (el(1) << 16), el(2) | (el(3) << 16)};
                    } else {
                        static_assert(NV == 8, "unsupported tile height");
                        *(u32x4*)dst = u32x4{el(0) | (el(1) << 16), el(2) | (el(3) << 16),
                                             el(4) | (el(5) << 16), el(6) | (el(7) << 16)};
                    }
                } else {
                    if constexpr (NV == 1) {
                        *(uint32_t*)dst = v[0][j];
                    } else if constexpr (NV == 2) {
                        *(u32x2*)dst = u32x2{v[0][j], v[1][j]};
                    } else if constexpr (NV == 4) {
                        *(u32x4*)dst = u32x4{v[0][j], v[1][j], v[2][j], v[3][j]};
                    } else {
                        static_assert(NV == 8, "unsupported tile height");
                        *(u32x4*)dst = u32x4{v[0][j], v[1][j], v[2][j], v[3][j]};
                        *(u32x4*)(dst + 16) = u32x4{v[4][j], v[5][j], v[6][j], v[7][j]};
                    }
                }
            }
        }
    }
};

// G > 1: the block is G groups of four wavefronts that take the k steps of the tile in turn (group g the steps
// g, g + G, ...), each with its own pair of stage buffers; their sums are added through LDS in a fixed order before
// the epilogue.  A product with fewer tiles than compute units then has G loads in flight per tile instead of
// one: its time is set by the latency of a step's loads, not by arithmetic.
// KW = 4: the four wavefronts of a group do not split the tile but the k of a step (each a quarter of it, on the
// whole tile), which lets the tile be as small as one 32x32 matrix instruction: the products of a 256 x 512 layer
// are then 128 tiles instead of 32, and a tile's arithmetic is spread over sixteen wavefronts.
template <typename T, int BM, int BN, int G = 1, int KW = 1>
__global__ __launch_bounds__(kGemmThreads * G) void gemm_tile_kernel(FLOP_HEAD_PARAMS, const GemmGroup grp)
{
    constexpr int ES = sizeof(T);
    constexpr int BK = kStepBytes / ES;
    static_assert(KW == 1 || KW == 4, "a step's k goes to one wavefront or to the group's four");
    constexpr int WGRID = KW == 1 ? 2 : 1;      // 2 x 2 wavefronts over the tile, or every wavefront on all of it
    constexpr int WTM = BM / WGRID, WTN = BN / WGRID;
    constexpr int TM = WTM / 32, TN = WTN / 32; // 32x32 MFMA tiles per wave
    static_assert(TM >= 1 && TN >= 1, "tile too small");
    constexpr int A_BYTES = BM * kLdsRow, B_BYTES = BN * kLdsRow;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    // ---- which problem, which tile -------------------------------------
    GemmProblem pr;
    int tile_m, tile_n;
    bool from_head;
    if (!(locate_tile<ES, BM, BN>(FLOP_HEAD_ARGS, grp, pr, tile_m, tile_n, from_head))) return;
    if (from_head) finish_problem(pr, grp.p[0]);   // (this kernel's loads need a_vec / b_vec at once)
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int group = (int)threadIdx.x / kGemmThreads;   // wave-uniform
    const int tid = (int)threadIdx.x % kGemmThreads;     // thread inside its group
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = KW == 1 ? wave >> 1 : 0, wn = KW == 1 ? wave & 1 : 0;
    const int l32 = lane & 31, lhi = lane >> 5;
    unsigned char* gmem = smem + group * 2 * (A_BYTES + B_BYTES);   // the group's two stage buffers

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    TileStager<ES, BM> sa;
    TileStager<ES, BN> sb;
    // every group makes the same number of passes (the barriers are the block's); a pass beyond K loads zeros
    const int nk = ((pr.K + BK - 1) / BK + G - 1) / G;

    sa.load(pr.A, pr.lda, pr.a_kmajor, pr.a_vec != 0, m0, group * BK, pr.M, pr.K, tid);
    sb.load(pr.B, pr.ldb, pr.b_kmajor, pr.b_vec != 0, n0, group * BK, pr.N, pr.K, tid, pr.b_map);
    sa.store(gmem, pr.a_kmajor, tid);
    sb.store(gmem + A_BYTES, pr.b_kmajor, tid);
    __syncthreads();

    for (int s = 0; s < nk; ++s) {
        unsigned char* cur = gmem + (s & 1) * (A_BYTES + B_BYTES);
        unsigned char* nxt = gmem + ((s + 1) & 1) * (A_BYTES + B_BYTES);
        const bool more = (s + 1 < nk);
        if (more) {
            sa.load(pr.A, pr.lda, pr.a_kmajor, pr.a_vec != 0, m0, ((s + 1) * G + group) * BK, pr.M, pr.K, tid);
            sb.load(pr.B, pr.ldb, pr.b_kmajor, pr.b_vec != 0, n0, ((s + 1) * G + group) * BK, pr.N, pr.K, tid, pr.b_map);
        }
        const unsigned char* la = cur + (wm * WTM + l32) * kLdsRow + lhi * 16;
        const unsigned char* lb = cur + A_BYTES + (wn * WTN + l32) * kLdsRow + lhi * 16;
#pragma unroll
        for (int cc = 0; cc < kStepBytes / 32 / KW; ++cc) {
            const int c = KW == 1 ? cc : wave;   // 32-byte piece of the step's k
            u32x4 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *(const u32x4*)(la + i * 32 * kLdsRow + c * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = *(const u32x4*)(lb + j * 32 * kLdsRow + c * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (ES == 2) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]),
                            acc[i][j], 0, 0, 0);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            // copy the lanes' words out before reinterpreting them
                            const uint32_t aw = af[i][e], bw = bf[j][e];
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                __builtin_bit_cast(float, aw), __builtin_bit_cast(float, bw),
                                acc[i][j], 0, 0, 0);
                        }
                    }
                }
        }
        if (more) {
            sa.store(nxt, pr.a_kmajor, tid);
            sb.store(nxt + A_BYTES, pr.b_kmajor, tid);
        }
        __syncthreads();
    }

    // ---- partial sums added in a fixed order (the loop ended with a barrier: the stage buffers are free).
    // Contributors: the G groups, times the group's four wavefronts when they split k; the first one collects.
    if constexpr (G > 1 || KW > 1) {
        float* part = (float*)smem;
        constexpr int OWNERS = KW == 1 ? kGemmThreads : 64;   // threads of a contributor, each with its own outputs
        constexpr int PER = TM * TN * 16 * OWNERS;
        constexpr int NCONTRIB = G * KW;
        const int cid = KW == 1 ? group : group * KW + wave;
        const int otid = KW == 1 ? tid : lane;
        if (cid > 0) {
            float* mine = part + (cid - 1) * PER + otid;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mine[((i * TN + j) * 16 + v) * OWNERS] = acc[i][j][v];
        }
        __syncthreads();
        if (cid > 0) return;
#pragma unroll 1
        for (int gg = 1; gg < NCONTRIB; ++gg) {   // not unrolled: 16 values in flight per thread are enough
            const float* theirs = part + (gg - 1) * PER + otid;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] += theirs[((i * TN + j) * 16 + v) * OWNERS];
        }
    }

    // ---- epilogue --------------------------------------------------------
    // Accumulator layout of the 32x32 MFMA: lane holds column (lane % 32) and
    // rows 8*(v/4) + 4*(lane/32) + v%4 for v = 0..15.
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + l32;
        if (col >= pr.N) continue;
        const float scale = pr.col_scale ? pr.col_scale[col] : 1.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                if (row < pr.M) {
                    const float val = acc[i][j][v] * scale;
                    const int64_t orow = pr.c_rowmap ? pr.c_rowmap[row] : row;
                    if constexpr (ES == 2)
                        ((uint16_t*)pr.C)[orow * pr.ldc + col] = (uint16_t)f32_to_bf16_bits(val);
                    else
                        ((float*)pr.C)[orow * pr.ldc + col] = val;
                }
            }
    }
}

template <int BM, int BN, int G = 1, int KW = 1>
constexpr size_t gemm_lds_bytes()
{
    const size_t stages = (size_t)G * 2 * (size_t)(BM + BN) * kLdsRow;
    const size_t partials = (size_t)(G * KW - 1) * BM * BN * sizeof(float);
    return stages > partials ? stages : partials;
}

}  // namespace flop
