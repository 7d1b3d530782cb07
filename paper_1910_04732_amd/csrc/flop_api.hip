// C-ABI entry points of the gated factorized layer library (see include/flop.h).
// Host side only validates arguments, picks tile shapes and enqueues kernels.
#include "../../include/flop.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <initializer_list>
#include <mutex>
#include <vector>

#include "gemm_tile.hip.h"
#include "gemm_dma.hip.h"
#include "gemm_lowrank.hip.h"
#include "stream_kernels.hip.h"
#include "embed_kernels.hip.h"
#include "bench_hooks.h"

using namespace flop;

namespace {

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline size_t elem_size(flop_dtype dt) { return dt == FLOP_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
inline bool valid_dtype(int dt) { return dt == FLOP_F32 || dt == FLOP_BF16; }
inline bool valid_hc(flop_hc hc) { return hc.l < 0.0f && hc.r > 1.0f && hc.beta > 0.0f; }
constexpr int64_t kMaxDim = (int64_t)1 << 30;
constexpr int64_t kMaxLd = (int64_t)1 << 32;   // leading dimensions beyond this are taken for a caller's mistake
inline bool ld_too_large(std::initializer_list<int64_t> lds)
{
    for (int64_t v : lds) if (v > kMaxLd) return true;
    return false;
}

// ------------------------------------------------------------------------
// Contraction launcher
// ------------------------------------------------------------------------
struct GemmDesc {
    const void* A; int64_t lda; bool a_kmajor;
    const void* B; int64_t ldb; bool b_kmajor;
    void* C; int64_t ldc;
    int64_t M, N, K;
    const float* col_scale;
    // run-time segment (see GemmProblem); all zero for the dense layer
    const int32_t* seg; int seg_dim; bool seg_a, seg_b, seg_c; const int32_t* c_rowmap;
    // fused column reduction sum_m C[m,n] * dot[m,n] per tile row (see GemmProblem); honoured by the
    // asynchronous-transfer kernel only
    const void* dot; int64_t lddot; float* dot_partial;
    // extent read on the device (see GemmProblem): 1 = M, 2 = K, 3 = N
    const int32_t* ext; int ext_dim;
    // k split (see GemmProblem); set by launch_group
    int ksplit; float* split_out;
    // gate computed in the epilogue instead of col_scale (see GemmProblem); only for products that
    // gate_fusable() accepts
    const float* gate_alpha; const float* gate_u; float gate_beta, gate_l, gate_r;
    // B gathered by an index list (see GemmProblem): rows of the b_map_rows-row matrix at B
    const int32_t* b_map; int64_t b_map_rows;
    // launch-wide (read from the first product): lay the products out over the XCDs one after another instead
    // of cutting every product into eight (see GemmGroup::contiguous); needs host-known extents and no k split
    bool few_xcds;
};

// Kernels that need more dynamic LDS than the default limit get the attribute once per device (a function's
// attributes belong to the device it is loaded on); which devices are done is a bit mask.
struct AttrOnce {
    std::atomic<uint64_t> devices{0};
    // true if the current device still needs the attribute; *dev receives the device
    bool needed(int* dev) const
    {
        if (hipGetDevice(dev) != hipSuccess) *dev = 0;
        return ((devices.load(std::memory_order_acquire) >> (*dev & 63)) & 1ull) == 0;
    }
    void done(int dev) { devices.fetch_or(1ull << (dev & 63), std::memory_order_release); }
};

#ifdef FLOP_PHASE_STAMPS
// Measurement build: launches of the transfer kernel take the stamp slots 0, 1, ... after flop_bench_phases_begin()
std::atomic<int> g_stamp_launches{kStampSlots};
#endif

// One launch of a tile kernel over up to kMaxGroup products.  Products are ordered
// by decreasing k extent so that the longest tiles are dispatched first.
// lds_extra: what a launch with a B gathered along k adds for its table (only such launches ask for it)
template <int ES, int BM, int BN>
int launch_tiles(void (*kernel)(FLOP_HEAD_PARAMS, const GemmGroup), size_t lds, AttrOnce* attr, int kernel_id, int threads,
                 const GemmDesc* d_in, int count, hipStream_t stream, const BoundaryRider* rider = nullptr,
                 bool* carried = nullptr, size_t lds_extra = 0)
{
    int dev = 0;
    if (attr->needed(&dev)) {
        if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(lds + lds_extra)) != hipSuccess)
            return FLOP_ERR_HIP;
        attr->done(dev);
    }
    bool k_gather = false;
    for (int i = 0; i < count; ++i) k_gather = k_gather || (d_in[i].b_map && !d_in[i].b_kmajor);
    if (k_gather) lds += lds_extra;
    if (lds > 160 * 1024) return FLOP_ERR_SHAPE;   // beyond a compute unit's LDS (no shape of this library reaches it)
    GemmDesc d[kMaxGroup];
    for (int i = 0; i < count; ++i) d[i] = d_in[i];
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && d[j].K > d[j - 1].K; --j) { GemmDesc t = d[j]; d[j] = d[j - 1]; d[j - 1] = t; }
    GemmGroup grp;
    memset(&grp, 0, sizeof(grp));
    int per_xcd_total = 0;
    double flops = 0.0;
    int tiles = 0;
    for (int i = 0; i < count; ++i) {
        GemmProblem& p = grp.p[i];
        p.A = d[i].A; p.B = d[i].B; p.C = d[i].C;
        p.col_scale = d[i].col_scale;
        p.gate_alpha = d[i].gate_alpha; p.gate_u = d[i].gate_u;
        p.gate_beta = d[i].gate_beta; p.gate_l = d[i].gate_l; p.gate_r = d[i].gate_r;
        p.seg = d[i].seg; p.seg_dim = d[i].seg_dim; p.seg_a = d[i].seg_a; p.seg_b = d[i].seg_b; p.seg_c = d[i].seg_c;
        p.c_rowmap = d[i].c_rowmap;
        p.dot = d[i].dot; p.lddot = d[i].lddot; p.dot_partial = d[i].dot_partial; p.dot_ld = d[i].N;
        p.ext = d[i].ext; p.ext_dim = d[i].ext_dim;
        p.ksplit = d[i].ksplit; p.split_out = d[i].split_out;
        p.b_map = d[i].b_map; p.b_map_rows = (int)d[i].b_map_rows;
        p.lda = d[i].lda; p.ldb = d[i].ldb; p.ldc = d[i].ldc;
        p.M = (int)d[i].M; p.N = (int)d[i].N; p.K = (int)d[i].K;
        p.tiles_m = (int)((d[i].M + BM - 1) / BM);
        p.tiles_n = (int)((d[i].N + BN - 1) / BN);
        p.xcd_begin = per_xcd_total;
        const int slices = d[i].ksplit > 1 ? d[i].ksplit : 1;
        p.tiles_per_xcd = (p.tiles_m * p.tiles_n * slices + 7) / 8;
        p.a_kmajor = d[i].a_kmajor; p.b_kmajor = d[i].b_kmajor;
        p.a_vec = aligned16(d[i].A) && (d[i].lda * ES) % 16 == 0;
        p.b_vec = aligned16(d[i].B) && (d[i].ldb * ES) % 16 == 0;
        per_xcd_total += p.tiles_per_xcd;
        tiles += p.tiles_m * p.tiles_n * slices;
        flops += 2.0 * (double)d[i].M * (double)d[i].N * (double)d[i].K;
    }
    grp.count = count;
    if (tiles == 0) return FLOP_OK;
    grp.tile_blocks = 8 * per_xcd_total;
    bool contiguous = count > 0 && d[0].few_xcds;
    for (int i = 0; i < count; ++i) contiguous = contiguous && !d[i].seg && !d[i].ext && d[i].ksplit <= 1;
    if (contiguous) {
        // Cut the sequence of all tiles (products in launch order) into eight pieces of equal work; a tile's work is
        // its 64-k steps plus what its first load and its store cost in steps.
        constexpr double kTileOverheadSteps = 8.0;
        double work[kMaxGroup], total = 0.0;
        int begin[kMaxGroup + 1];
        begin[0] = 0;
        for (int i = 0; i < count; ++i) {
            const int t = grp.p[i].tiles_m * grp.p[i].tiles_n;
            work[i] = (double)((d[i].K + 63) / 64) + kTileOverheadSteps;
            total += work[i] * t;
            begin[i + 1] = begin[i] + t;
            grp.p[i].xcd_begin = begin[i];
        }
        grp.contiguous = 1;
        grp.xcd_first[0] = 0;
        int longest = 0;
        for (int x = 1; x <= 8; ++x) {
            const double target = total * x / 8.0;
            double cum = 0.0;
            int pos = begin[count];
            for (int i = 0; i < count; ++i) {
                const double w = work[i] * (begin[i + 1] - begin[i]);
                if (cum + w >= target) { pos = begin[i] + (int)((target - cum) / work[i] + 0.5); break; }
                cum += w;
            }
            if (x == 8 || pos > begin[count]) pos = begin[count];
            if (pos < grp.xcd_first[x - 1]) pos = grp.xcd_first[x - 1];
            grp.xcd_first[x] = pos;
            longest = pos - grp.xcd_first[x - 1] > longest ? pos - grp.xcd_first[x - 1] : longest;
        }
        grp.tile_blocks = 8 * longest;
    }
    if (rider) {   // extra blocks behind the tiles do the step-boundary work
        grp.rider = *rider;
        grp.rider_blocks = rider->bx * (rider->count + 1);
        if (carried) *carried = true;
    }
    // the launch head (see LaunchHead): the first product as scalar arguments, when it is a plain one
    LaunchHead head = {};
    const GemmDesc& d0 = d[0];
    if (!contiguous && !d0.seg && !d0.ext && !d0.b_map && d0.ksplit <= 1 && d0.lda <= 0xFFFFFFFFll && d0.ldb <= 0xFFFFFFFFll &&
        grp.p[0].tiles_m * grp.p[0].tiles_n > 0) {
        head.A = d0.A; head.B = d0.B;
        head.lda = (uint32_t)d0.lda; head.ldb = (uint32_t)d0.ldb;
        head.M = (int)d0.M; head.N = (int)d0.N; head.K = (int)d0.K;
        head.flags = kHeadValid | (d0.a_kmajor ? kHeadAKmajor : 0) | (d0.b_kmajor ? kHeadBKmajor : 0);
        head.next = grp.p[0].tiles_per_xcd;
    }
#ifdef FLOP_PHASE_STAMPS
    grp.stamp_slot = -1;
    if (kernel_id % 1000 >= 100) {   // the transfer kernel
        const int slot = g_stamp_launches.fetch_add(1);
        if (slot < kStampSlots) grp.stamp_slot = slot;
    }
#endif
    const dim3 grid((unsigned)(grp.tile_blocks + grp.rider_blocks));
    TraceSlot* ts = trace_acquire(kernel_id, tiles, flops);
    if (ts)   // the dispatch itself stamps the two events at kernel begin and end
        hipExtLaunchKernelGGL(kernel, grid, dim3((unsigned)threads), lds, stream, ts->start, ts->stop, 0, head.A, head.B,
                              head.lda, head.ldb, head.M, head.N, head.K, head.flags, head.next, grp);
    else
        hipLaunchKernelGGL(kernel, grid, dim3((unsigned)threads), lds, stream, head.A, head.B, head.lda, head.ldb, head.M,
                           head.N, head.K, head.flags, head.next, grp);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

inline int64_t count_tiles(const GemmDesc* d, int count, int bm, int bn);

template <typename T, int B, int G = 1, int KW = 1>
int launch_generic_groups(const GemmDesc* d, int count, hipStream_t stream)
{
    static AttrOnce attr;
    return launch_tiles<sizeof(T), B, B>(gemm_tile_kernel<T, B, B, G, KW>, gemm_lds_bytes<B, B, G, KW>(), &attr,
                                         (sizeof(T) == 2 ? 1000 : 0) + B + 10000 * (G - 1), kGemmThreads * G, d, count, stream);
}

// Generic kernel.  A launch of 64x64 tiles that leaves half of the compute units without a tile while every tile
// has at least 8 steps lasts as long as one tile's chain of load latencies and its own arithmetic on one unit: it
// runs on 32x32 tiles instead, in blocks of four k groups (1024 threads) with each step's k split over a group's
// wavefronts (C1's products: 128 to 384 blocks instead of 32 to 96; 64x64 tiles with four k groups measured
// 21 us per backward launch against 13).
template <typename T, int B>
int launch_generic(const GemmDesc* d, int count, hipStream_t stream)
{
    if constexpr (B == 64) {
        constexpr int BK = kStepBytes / (int)sizeof(T);
        int64_t min_k = INT64_MAX;
        bool fixed = true;
        for (int i = 0; i < count; ++i) {
            if (d[i].M <= 0 || d[i].N <= 0) continue;
            min_k = d[i].K < min_k ? d[i].K : min_k;
            fixed = fixed && !(d[i].seg || d[i].ext);
        }
        if (fixed && min_k != INT64_MAX && min_k >= 8 * BK) {
            if (count_tiles(d, count, 64, 64) <= 128) return launch_generic_groups<T, 32, 4, 4>(d, count, stream);
        }
    }
    return launch_generic_groups<T, B, 1>(d, count, stream);
}

// Block shapes of the bf16 transfer kernel (see TileShape): tile, stage buffers, wave grid, k groups.
using Shape128x128 = TileShape<128, 128, 2, 2, 2, 1>;     // 64 KB, two blocks per compute unit
using Shape128x64 = TileShape<128, 64, 3, 2, 2, 1>;       // 72 KB
using Shape64x64 = TileShape<64, 64, 3, 2, 2, 1>;         // 48 KB, three blocks per compute unit
using Shape64x64g2 = TileShape<64, 64, 3, 2, 2, 2>;       // 96 KB, 512 threads: few tiles, long contraction
using Shape64x96g2 = TileShape<64, 96, 3, 2, 3, 2>;       // 144 KB, 768 threads: 256 equal tiles on 2048 x 768
using Shape128x64g2 = TileShape<128, 64, 3, 2, 2, 2>;     // 144 KB, 512 threads
using Shape128x128g2 = TileShape<128, 128, 2, 2, 2, 2>;   // 128 KB, 512 threads
using Shape256x128 = TileShape<256, 128, 3, 4, 2, 1>;     // 144 KB, 512 threads: 85 flop per staged byte
using Shape64x64g4 = TileShape<64, 64, 2, 2, 2, 4>;       // 128 KB, 1024 threads
using Shape64x96 = TileShape<64, 96, 3, 2, 3, 1>;         // 72 KB, 384 threads
using Shape64x64g2n2 = TileShape<64, 64, 2, 2, 2, 2>;     // 64 KB, 512 threads, two blocks per compute unit
using Shape64x96g2n2 = TileShape<64, 96, 2, 2, 3, 2>;     // 96 KB, 768 threads
using Shape128x64g2n2 = TileShape<128, 64, 2, 2, 2, 2>;   // 96 KB, 512 threads
using Shape64x64n2 = TileShape<64, 64, 2, 2, 2, 1>;       // 32 KB, five blocks per compute unit
constexpr int kNumShapes = kNumTileShapes;
struct ShapeInfo { int bm, bn, groups; };
constexpr ShapeInfo kShapes[kNumShapes] = {
    {128, 128, 1}, {128, 64, 1}, {64, 64, 1}, {64, 64, 2}, {64, 96, 2}, {128, 64, 2}, {128, 128, 2},
    {256, 128, 1}, {64, 64, 4}, {64, 96, 1}, {64, 64, 2}, {64, 96, 2}, {128, 64, 2}, {64, 64, 1},
};

template <typename SH, bool BKM, int XFER>
int launch_dma(const GemmDesc* d, int count, hipStream_t stream, const BoundaryRider* rider, bool* carried)
{
    static AttrOnce attr;
    return launch_tiles<2, SH::BM, SH::BN>(gemm_bf16_dma_kernel<SH, BKM, XFER>, gemm_dma_lds_bytes<SH>(), &attr,
                                           1100 + (SH::BM + SH::BN) / 2 + 10000 * (SH::G - 1), SH::THREADS, d, count,
                                           stream, rider, carried, (!BKM && XFER == 16) ? (size_t)kKtabBytes : 0);
}

// The DMA kernel describes each operand with a buffer descriptor whose range is below 2 GiB.  For a
// k-contiguous operand the descriptor starts at the tile's first row, so only 128 rows have to fit; for a
// [k][row] operand it spans the whole k range of the tile, and a larger operand is cut into k slices
// (float32 partial products, added by a second kernel) until every slice fits.
constexpr int64_t kDescLimit = ((int64_t)1 << 31) - 65536;
constexpr int kMaxSlices = 16;

// Fewest k slices with which a [k][row] operand of `rows` columns, K rows and leading dimension ld fits;
// 0 if even kMaxSlices do not.  The slicing is the kernel's: ceil(steps / s) steps of 64 per slice.
inline int slices_to_fit(int64_t ld, int64_t rows, int64_t K)
{
    const int64_t steps = (K + 63) / 64;
    for (int sl = 1; sl <= kMaxSlices; ++sl) {
        int64_t chunk = ((steps + sl - 1) / sl) * 64;
        if (chunk > K) chunk = K;
        if (((chunk - 1) * ld + round_up(rows, 8)) * 2 < kDescLimit) return sl;
    }
    return 0;
}

// Transfer width in bytes the DMA kernel can use for a product (16 when bases are 16-byte aligned and
// leading dimensions are multiples of 8 elements, else 4 when bases are 4-byte aligned and leading
// dimensions even), 0 if the product needs the generic kernel; *min_split = k slices it must be cut into.
int dma_width(const GemmDesc& g, int* min_split)
{
    auto align = [](const void* p, int64_t ld) {
        if (aligned16(p) && ld % 8 == 0) return 16;
        if (((uintptr_t)p & 3u) == 0 && ld % 2 == 0) return 4;
        return 0;
    };
    *min_split = 1;
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return 0;
    int need = 1;
    auto fits = [&](bool kmajor, int64_t ld, int64_t rows) {
        if (kmajor) return ((rows < 128 ? rows : 128) - 1) * ld + round_up(g.K, 8) < kDescLimit / 2;
        const int sl = slices_to_fit(ld, rows, g.K);
        if (sl > need) need = sl;
        return sl > 0;
    };
    if (!fits(g.a_kmajor, g.lda, g.M)) return 0;
    if (g.b_map) {   // a gathered B is described whole, and its k rows by 16-bit entries of a table of kKtabMaxK
        if (((g.b_map_rows - 1) * g.ldb + round_up(g.b_kmajor ? g.K : g.N, 8)) * 2 >= kDescLimit) return 0;
        if (!g.b_kmajor && (g.K > kKtabMaxK || g.b_map_rows >= (int64_t)kKtabNone)) return 0;
    } else if (!fits(g.b_kmajor, g.ldb, g.N)) return 0;
    *min_split = need;
    const int wa = align(g.A, g.lda), wb = align(g.B, g.ldb);
    const int w = wa < wb ? wa : wb;
    return (g.b_map && w != 16) ? 0 : w;   // gathered operands: 16-byte transfers or the generic kernel
}

inline int64_t count_tiles(const GemmDesc* d, int count, int bm, int bn)
{
    int64_t t = 0;
    for (int i = 0; i < count; ++i) t += ((d[i].M + bm - 1) / bm) * ((d[i].N + bn - 1) / bn);
    return t;
}

// Slices for a product with few tiles and a long k extent (weight-gradient and wide-output
// shapes): enough blocks to fill the chip, at least 16 steps of 64 k each.  Depends on the
// shape only, so that the workspace can be sized without knowing the launch.
inline int plan_ksplit(int64_t M, int64_t N, int64_t K)
{
    const int64_t t = ((M + 127) / 128) * ((N + 63) / 64);
    const int64_t steps = (K + 63) / 64;
    if (t >= 256 || steps < 64) return 1;
    int64_t s = (512 + t - 1) / t;
    if (s > steps / 16) s = steps / 16;
    if (s > kMaxSlices) s = kMaxSlices;
    return s < 2 ? 1 : (int)s;
}

// Block shape for a launch.  Generic kernel (xfer == 0): 128x128 (0) when that still gives every compute unit
// work, else 64x64 (2).  bf16 transfer kernel: whichever candidate a small timing model of the launch puts
// first.  The model follows one compute unit: tiles are numbered by decreasing k extent (as the kernel numbers
// them) and dealt to the 256 units in turn; a unit runs up to `occ` blocks at once; a block advances one 64-k
// step (of each of its k groups) in max(lat_us, bytes staged per step by the unit's running blocks / intake rate)
// and pays tile_us once for its first load and its output store.  The intake rate (130 KB/us per unit) and the
// per-shape constants were fitted to per-launch times of the eight launches of the BERT-shaped step and the
// sixteen of a 410-wide Transformer layer, measured with every shape forced in turn; what the model decides in
// practice: one round of large tiles beats two
// rounds of smaller ones, a product with few tiles and a long k extent wants small tiles or k groups, launches
// of many rounds want the largest tile.
struct ShapeModel { int cfg, bm, bn, groups, occ; double lat_us, tile_us; };
constexpr ShapeModel kShapeModels[] = {
    {2, 64, 64, 1, 3, 0.20, 2.0},   {9, 64, 96, 1, 2, 0.20, 3.0},   {3, 64, 64, 2, 1, 0.22, 2.5},  {4, 64, 96, 2, 1, 0.40, 3.0},
    {1, 128, 64, 1, 2, 0.24, 3.0},  {0, 128, 128, 1, 2, 0.52, 4.5}, {7, 256, 128, 1, 1, 0.54, 4.5},
};
constexpr double kIntakeKBPerUs = 130.0;

inline double model_launch_us(const ShapeModel& sm, const GemmDesc* d, const int* order, int count)
{
    const double stage_kb = (double)(sm.bm + sm.bn) * 128.0 * sm.groups / 1024.0;
    const double tile_steps = sm.tile_us / sm.lat_us;
    double active[8];
    int nactive = 0;
    double t = 0.0;
    int oi = 0;
    int64_t index = 0, prod_end = 0, next_mine = 0;   // global tile index; unit 0 owns every 256th tile
    double prod_steps = 0.0;
    bool more = true;
    while (more || nactive > 0) {
        while (nactive < sm.occ && more) {
            // advance to the product that holds tile next_mine
            while (next_mine >= prod_end) {
                if (oi >= count) { more = false; break; }
                const GemmDesc& g = d[order[oi++]];
                if (g.M <= 0 || g.N <= 0) continue;
                const int slices = (g.seg || g.ext || g.b_map) ? 1 : plan_ksplit(g.M, g.N, g.K);
                int64_t steps = (((g.K + 63) / 64) + slices - 1) / slices;
                steps = (steps + sm.groups - 1) / sm.groups;
                prod_steps = (double)(steps > 0 ? steps : 1) + tile_steps;
                index = prod_end;
                prod_end = index + ((g.M + sm.bm - 1) / sm.bm) * ((g.N + sm.bn - 1) / sm.bn) * slices;
            }
            if (!more) break;
            active[nactive++] = prod_steps;
            next_mine += 256;
        }
        if (nactive == 0) break;
        const double by_intake = (double)nactive * stage_kb / kIntakeKBPerUs;
        const double step_us = sm.lat_us > by_intake ? sm.lat_us : by_intake;
        double adv = active[0];
        for (int i = 1; i < nactive; ++i) adv = active[i] < adv ? active[i] : adv;
        t += adv * step_us;
        int keep = 0;
        for (int i = 0; i < nactive; ++i) {
            const double left = active[i] - adv;
            if (left > 1e-9) active[keep++] = left;
        }
        nactive = keep;
    }
    return t;
}

// xfer: 16 or 4 for the bf16 transfer kernel (4-byte transfers run the three shapes of four wavefronts), 0 for
// the generic kernel
inline int pick_cfg(const GemmDesc* d, int count, int xfer)
{
    if (xfer && forced_tile_shape() >= 0) return forced_tile_shape();   // flop_bench.h
    bool narrow = true;   // no product wider than 64 columns: wider tiles would be mostly empty
    for (int i = 0; i < count; ++i) narrow = narrow && d[i].N <= 64;
    if (!xfer) {
        const int64_t t128 = count_tiles(d, count, 128, 128);
        return (t128 >= 320 && !narrow) ? 0 : 2;
    }
    // Extents that only the device knows (token segments of the embedding: the host sees upper bounds) defeat the
    // model: large tiles when even the bounds give more than a round of them, else the smallest
    bool segmented = false;
    for (int i = 0; i < count; ++i) segmented = segmented || d[i].seg != nullptr;
    if (segmented) return (count_tiles(d, count, 128, 128) >= 320 && !narrow) ? 0 : 2;
    int order[kMaxGroup];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && d[order[j]].K > d[order[j - 1]].K; --j) { int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t; }
    // Where the fitted constants cannot be trusted (they come from launches of one round of tiles): k groups
    // only pay on a long contraction; 96-wide tiles only where they waste no columns; with one 256x128 block per
    // unit nothing hides a tile's first load and store, so that shape needs a single round or long tiles
    int64_t min_steps = INT64_MAX, max_steps = 0;
    bool n96 = true;
    for (int i = 0; i < count; ++i) {
        if (d[i].M <= 0 || d[i].N <= 0) continue;
        const int64_t st = (d[i].K + 63) / 64;
        min_steps = st < min_steps ? st : min_steps;
        max_steps = st > max_steps ? st : max_steps;
        n96 = n96 && d[i].N % 96 == 0;
    }
    const int64_t t256 = count_tiles(d, count, 256, 128);
    // many rounds of long tiles: the launch runs at the chip's power limit, where the shape that moves the fewest
    // bytes per flop wins (measured 3-6 % over 128x128 on 8192 x 3056 x 3056 .. 9168 products), whatever the
    // model of a lightly loaded unit says
    if (xfer == 16 && !narrow && t256 >= 768 && min_steps >= 32) return 7;
    int best = 2;
    double best_t = 0.0;
    bool first = true;
    for (const ShapeModel& sm : kShapeModels) {   // from small to large tiles: a larger one wins ties (fewer bytes moved)
        if (narrow && sm.bn > 64) continue;
        if (xfer == 4 && !(sm.cfg <= 2)) continue;
        if (sm.groups > 1 && max_steps < 32) continue;
        if (sm.bn == 96 && !n96) continue;
        if (sm.bm == 256 && !(t256 <= 256 || min_steps >= 32)) continue;
        const double t = model_launch_us(sm, d, order, count);
        if (first || t <= best_t * 1.01) { best = sm.cfg; best_t = first || t < best_t ? t : best_t; first = false; }
    }
    return best;
}

inline size_t split_bytes_for(int slices, int64_t M, int64_t N)
{
    return slices > 1 ? (size_t)round_up((int64_t)slices * M * N * 4, 256) : 0;
}
// Scratch of one product as the workspace queries size it: the split that pays, or the one that densely
// stored [k][row] operands (leading dimensions lda_rows / ldb_rows, 0 for a k-contiguous operand) force.
inline size_t ksplit_bytes(int64_t M, int64_t N, int64_t K, int64_t lda_rows = 0, int64_t ldb_rows = 0)
{
    int s = plan_ksplit(M, N, K);
    if (lda_rows > 0) { const int f = slices_to_fit(lda_rows, M, K); if (f > s) s = f; }
    if (ldb_rows > 0) { const int f = slices_to_fit(ldb_rows, N, K); if (f > s) s = f; }
    return split_bytes_for(s, M, N);
}

template <bool BKM, int XFER>
int launch_dma_cfg(int cfg, const GemmDesc* d, int count, hipStream_t stream, const BoundaryRider* rider, bool* carried)
{
    if constexpr (XFER == 16) {
        switch (cfg) {
            case 3: return launch_dma<Shape64x64g2, BKM, 16>(d, count, stream, rider, carried);
            case 4: return launch_dma<Shape64x96g2, BKM, 16>(d, count, stream, rider, carried);
            case 5: return launch_dma<Shape128x64g2, BKM, 16>(d, count, stream, rider, carried);
            case 6: return launch_dma<Shape128x128g2, BKM, 16>(d, count, stream, rider, carried);
            case 7: return launch_dma<Shape256x128, BKM, 16>(d, count, stream, rider, carried);
            case 8: return launch_dma<Shape64x64g4, BKM, 16>(d, count, stream, rider, carried);
            case 9: return launch_dma<Shape64x96, BKM, 16>(d, count, stream, rider, carried);
            case 10: return launch_dma<Shape64x64g2n2, BKM, 16>(d, count, stream, rider, carried);
            case 11: return launch_dma<Shape64x96g2n2, BKM, 16>(d, count, stream, rider, carried);
            case 12: return launch_dma<Shape128x64g2n2, BKM, 16>(d, count, stream, rider, carried);
            case 13: return launch_dma<Shape64x64n2, BKM, 16>(d, count, stream, rider, carried);
            default: break;
        }
    }
    switch (cfg) {   // rows that are only 4-byte aligned take the three shapes of four wavefronts
        case 0: case 6: case 7: return launch_dma<Shape128x128, BKM, XFER>(d, count, stream, rider, carried);
        case 1: case 5: case 12: return launch_dma<Shape128x64, BKM, XFER>(d, count, stream, rider, carried);
        default: return launch_dma<Shape64x64, BKM, XFER>(d, count, stream, rider, carried);
    }
}
// Tile rows of the shape that launch_dma_cfg<., XFER> runs for cfg
inline int cfg_tile_rows(int cfg, int xfer)
{
    if (xfer == 16) return kShapes[cfg].bm;
    return (cfg == 0 || cfg == 6 || cfg == 7 || cfg == 1 || cfg == 5 || cfg == 12) ? 128 : 64;
}

// Whether the store-bound kernel for ranks up to 256 takes the product: k-contiguous operands and 16-byte rows
// everywhere, a plain epilogue, and enough output that stores, not launch latencies, set the time: 8 M elements
// up to rank 64 (measured 1.25x the general kernel at 25 M outputs, 2.3x at 270 M); 64 M elements above, where
// a tile brings more bytes of B per byte stored (rank 128: 1.15x at 75 M outputs, 2x at 270 M, a loss at 25 M;
// rank 192: 1.35x at 75 M, 1.9x at 270 M; rank 256: 1.05x and 1.6x; at rank 306 - 320 the same design lost at 75 M).
inline bool lowrank_fits(const GemmDesc& g)
{
    const int64_t least = g.K <= 64 ? ((int64_t)1 << 23) : ((int64_t)1 << 26);
    return g.a_kmajor && g.b_kmajor && g.K > 0 && g.K <= kLrMaxK &&
           aligned16(g.A) && aligned16(g.B) && aligned16(g.C) && g.lda % 8 == 0 && g.ldb % 8 == 0 && g.ldc % 8 == 0 &&
           !g.col_scale && !g.gate_alpha && !g.seg && !g.ext && !g.dot_partial && !g.c_rowmap && g.ksplit <= 1 &&
           g.M > 0 && g.N > 0 && g.M * g.N >= least;
}

int launch_lowrank(const GemmDesc& g, hipStream_t stream)
{
    // variant by contraction extent: (k chunks, tile columns)
    const int variant = g.K <= 64 ? 0 : g.K <= 128 ? 1 : g.K <= 192 ? 2 : 3;
    static const int kc_of[4] = {4, 8, 12, 16}, cols_of[4] = {64, 64, 32, 32};
    const int cols = cols_of[variant];
    LowRankProblem pr;
    pr.A = (const uint16_t*)g.A; pr.B = (const uint16_t*)g.B; pr.C = (uint16_t*)g.C;
    pr.lda = g.lda; pr.ldb = g.ldb; pr.ldc = g.ldc;
    pr.M = (int)g.M; pr.N = (int)g.N; pr.K = (int)g.K;
    pr.bands = (int)((g.M + kLrRows - 1) / kLrRows);
    pr.tiles_n = (int)((g.N + cols - 1) / cols);
    // Eight tiles per block where that still fills the chip.  Short walks keep the blocks that run at the same
    // time on a few row bands, so that memory sees long runs of each row of C (1.2x the rate of long walks
    // that spread the same blocks over every row); the block's set-up is small beside eight tiles.
    for (int per = 8; ; per /= 2) {
        pr.splits = (int)round_up((pr.tiles_n + per - 1) / per, 8);
        pr.tiles_per_split = per;
        if (per == 1 || (int64_t)pr.splits * pr.bands >= 1024) break;
    }
    const int64_t blocks = (int64_t)pr.splits * pr.bands;
    if (blocks > (1 << 30)) return FLOP_ERR_SHAPE;
    TraceSlot* ts = trace_acquire(1300, pr.bands * pr.tiles_n, 2.0 * (double)g.M * (double)g.N * (double)g.K);
    void (*kernel)(const LowRankProblem) =
        variant == 0 ? gemm_bf16_lowrank_kernel<4, 64> : variant == 1 ? gemm_bf16_lowrank_kernel<8, 64> :
        variant == 2 ? gemm_bf16_lowrank_kernel<12, 32> : gemm_bf16_lowrank_kernel<16, 32>;
    const dim3 threads(lr_threads(kc_of[variant]));
    if (ts)
        hipExtLaunchKernelGGL(kernel, dim3((unsigned)blocks), threads, 0, stream, ts->start, ts->stop, 0, pr);
    else
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), threads, 0, stream, pr);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

// Whether a single bfloat16 product launched without split scratch runs on the asynchronous-transfer kernel
// unsplit - the only path that can compute the gate in its epilogue and carry riders.
bool gate_fusable(flop_dtype dt, const GemmDesc& g)
{
    if (dt != FLOP_BF16 || g.M <= 0 || g.N <= 0 || g.K <= 0 || g.seg || g.ext) return false;
    int min_split = 1;
    return dma_width(g, &min_split) != 0 && min_split == 1;
}

// rider / carried (nullable): step-boundary work to append to the launch; *carried is set if it went along
// (only the asynchronous-transfer kernel takes riders).
int launch_group(flop_dtype dt, const GemmDesc* d_in, int count, hipStream_t stream, int* fused_tile_rows = nullptr,
                 void* split_ws = nullptr, size_t split_bytes = 0, const BoundaryRider* rider = nullptr,
                 bool* carried = nullptr)
{
    const GemmDesc* d = d_in;
    if (fused_tile_rows) *fused_tile_rows = 0;
    if (dt == FLOP_BF16 && count == 1 && lowrank_fits(d[0])) return launch_lowrank(d[0], stream);
    if (dt == FLOP_BF16) {
        // the DMA kernel fixes the layout of B per launch; A may differ between the products
        int xfer = 16;
        int min_split[kMaxGroup];
        for (int i = 0; i < kMaxGroup; ++i) min_split[i] = 1;
        for (int i = 0; i < count; ++i) {
            const int w = d[i].b_kmajor == d[0].b_kmajor ? dma_width(d[i], &min_split[i]) : 0;
            xfer = w < xfer ? w : xfer;
        }
        const int cfg = pick_cfg(d, count, xfer);
        // k slices per product: what pays on short tile lists, at least what the operand sizes force
        GemmDesc ds[kMaxGroup];
        size_t used = 0;
        bool any_split = false, dot_lost = false;
        for (int i = 0; i < count && xfer; ++i) {
            ds[i] = d[i];
            const bool fixed_extents = !(ds[i].seg || ds[i].ext || ds[i].b_map);
            int sl = fixed_extents ? plan_ksplit(ds[i].M, ds[i].N, ds[i].K) : 1;
            if (sl > 1 && !(split_ws && used + split_bytes_for(sl, ds[i].M, ds[i].N) <= split_bytes)) sl = 1;
            if (sl < min_split[i]) {
                sl = min_split[i];
                if (!fixed_extents || !split_ws || used + split_bytes_for(sl, ds[i].M, ds[i].N) > split_bytes) xfer = 0;
            }
            if (sl > 1 && xfer) {
                ds[i].ksplit = sl;
                ds[i].split_out = (float*)((char*)split_ws + used);
                used += split_bytes_for(sl, ds[i].M, ds[i].N);
                any_split = true;
                if (ds[i].dot_partial) { ds[i].dot_partial = nullptr; dot_lost = true; }   // sums need the finished tile
            }
        }
        if (xfer) {
            if (fused_tile_rows && !dot_lost) *fused_tile_rows = cfg_tile_rows(cfg, xfer);
            int rc;
            if (xfer == 16) rc = ds[0].b_kmajor ? launch_dma_cfg<true, 16>(cfg, ds, count, stream, rider, carried) : launch_dma_cfg<false, 16>(cfg, ds, count, stream, rider, carried);
            else rc = ds[0].b_kmajor ? launch_dma_cfg<true, 4>(cfg, ds, count, stream, rider, carried) : launch_dma_cfg<false, 4>(cfg, ds, count, stream, rider, carried);
            if (rc != FLOP_OK || !any_split) return rc;
            for (int i = 0; i < count; ++i) {
                if (ds[i].ksplit <= 1) continue;
                int64_t blocks = (ds[i].M * ds[i].N + kStreamThreads * 4 - 1) / (kStreamThreads * 4);
                if (blocks > 4096) blocks = 4096;
                hipLaunchKernelGGL(splitk_reduce_kernel<2>, dim3((unsigned)blocks), dim3(kStreamThreads), 0, stream,
                                   (const float*)ds[i].split_out, ds[i].ksplit, ds[i].M, ds[i].N, ds[i].col_scale,
                                   ds[i].C, ds[i].ldc);
                if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
            }
            return FLOP_OK;
        }
        for (int i = 0; i < count; ++i)
            if (d[i].gate_alpha) return FLOP_ERR_HIP;   // callers check gate_fusable() first
        return pick_cfg(d, count, 0) == 0 ? launch_generic<uint16_t, 128>(d, count, stream) : launch_generic<uint16_t, 64>(d, count, stream);
    }
    for (int i = 0; i < count; ++i)
        if (d[i].gate_alpha) return FLOP_ERR_HIP;
    return pick_cfg(d, count, 0) == 0 ? launch_generic<float, 128>(d, count, stream) : launch_generic<float, 64>(d, count, stream);
}

// bwd workspace layout: [dh: n x ldh elements][partial: ceil(n/32) x r floats][k-split scratch of one phase]
// Rows of dh start on 128-byte boundaries once they are longer than that: a 64-k chunk of a row (128 bytes of
// bfloat16) then lies in one cache line instead of straddling two, which wide matrices feel (3056-wide: +15 %).
inline int64_t bwd_ldh(int64_t r, flop_dtype dt)
{
    const int64_t es = (int64_t)elem_size(dt);
    return round_up(r, (r * es > 128 ? 128 : 16) / es);
}
inline size_t bwd_dh_bytes(int64_t n, int64_t r, flop_dtype dt)
{
    return (size_t)round_up(n * bwd_ldh(r, dt) * (int64_t)elem_size(dt), 256);
}

inline size_t bwd_partial_bytes(int64_t n, int64_t r)
{
    return (size_t)round_up(((n + kColsumChunkRows - 1) / kColsumChunkRows) * r * 4, 256);
}
inline size_t bwd_split_bytes(int64_t n, int64_t d, int64_t r, int64_t dout)
{
    // [k][row] operands: P in dh = dy P; dy and g in dP = dy^T g; dh and x in dQ = dh^T x; Q in dx = dh Q
    const int64_t ldh = bwd_ldh(r, FLOP_BF16);
    const size_t ph1 = ksplit_bytes(n, r, dout, 0, r) + ksplit_bytes(dout, r, n, dout, r);
    const size_t ph2 = ksplit_bytes(r, d, n, ldh, d) + ksplit_bytes(n, d, r, 0, d);
    return ph1 > ph2 ? ph1 : ph2;
}
inline size_t fwd_split_bytes(int64_t n, int64_t d, int64_t r, int64_t dout)
{
    const size_t a = ksplit_bytes(n, r, d), b = ksplit_bytes(n, dout, r);
    return a > b ? a : b;
}

// ------------------------------------------------------------------------
// Embedding path: layout of the buffer saved between forward and backward, and
// of the backward workspace.  Sections are 256-byte aligned.
// ------------------------------------------------------------------------
struct EmbedLayout {
    size_t seg, perm, rows, run_start, uniq_ids, run_id, g[kEmbedMaxClusters], saved_total;
    size_t dy_sorted, dh[kEmbedMaxClusters], partial[kEmbedMaxClusters], scatter_head, scatter_tail, ws_total;
    int64_t ldg[kEmbedMaxClusters], ldds, ld_scatter;
};

inline EmbedLayout embed_layout(flop_dtype dt, int64_t n, int64_t d, int n_clusters, const int64_t* dims)
{
    EmbedLayout L;
    const int64_t es = (int64_t)elem_size(dt), vec = 16 / es;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (size_t)round_up((int64_t)bytes, 256); return o; };
    L.seg = take(kSegInts * 4);
    L.perm = take((size_t)n * 4);
    L.rows = take((size_t)n * 4);
    L.run_start = take((size_t)(n + 1) * 4);
    L.uniq_ids = take((size_t)n * 8);
    L.run_id = take((size_t)n * 4);
    for (int c = 0; c < n_clusters; ++c) {
        L.ldg[c] = round_up(dims[c], vec);
        L.g[c] = take((size_t)(n * L.ldg[c] * es));
    }
    L.saved_total = off;
    off = 0;
    L.ldds = round_up(d, vec);
    L.dy_sorted = take((size_t)(n * L.ldds * es));
    const int64_t chunks = (n + kColsumChunkRows - 1) / kColsumChunkRows;
    for (int c = 0; c < n_clusters; ++c) {
        L.dh[c] = take((size_t)(n * L.ldg[c] * es));
        L.partial[c] = take((size_t)(chunks * dims[c] * 4));
    }
    // window partial sums of the embedding gradient: one row of the widest cluster per window, twice
    L.ld_scatter = 0;
    for (int c = 0; c < n_clusters; ++c) L.ld_scatter = dims[c] > L.ld_scatter ? dims[c] : L.ld_scatter;
    const int64_t windows = (n + kScatterWindow - 1) / kScatterWindow;
    L.scatter_head = take((size_t)(windows * L.ld_scatter * 4));
    L.scatter_tail = take((size_t)(windows * L.ld_scatter * 4));
    L.ws_total = off;
    return L;
}

// Upper bounds of the two sizes from the sum of the cluster dimensions alone
// (what flop_workspace_bytes can know): every section may lose < 256 bytes to
// alignment and every dimension < 8 elements to rounding.
inline size_t embed_saved_bound(flop_dtype dt, int64_t n, int64_t dim_sum)
{
    const int64_t es = (int64_t)elem_size(dt);
    return (size_t)(kSegInts * 4 + n * 4 * 3 + (n + 1) * 4 + n * 8 + n * (dim_sum + 8 * kEmbedMaxClusters) * es +
                    256 * (6 + kEmbedMaxClusters));
}
inline size_t embed_ws_bound(flop_dtype dt, int64_t n, int64_t d, int64_t dim_sum)
{
    const int64_t es = (int64_t)elem_size(dt);
    const int64_t chunks = (n + kColsumChunkRows - 1) / kColsumChunkRows;
    const int64_t windows = (n + kScatterWindow - 1) / kScatterWindow;
    return (size_t)(n * (d + 8) * es + n * (dim_sum + 8 * kEmbedMaxClusters) * es + chunks * dim_sum * 4 +
                    2 * windows * dim_sum * 4 + 256 * (3 + 2 * kEmbedMaxClusters));
}

int validate_embed(flop_dtype dt, int64_t n_tokens, int32_t n_clusters, const flop_embed_cluster* cl, int64_t d,
                   int64_t* dims)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n_tokens < 0 || n_tokens > kEmbedMaxTokens || d <= 0 || d > kMaxDim) return FLOP_ERR_SHAPE;
    if (n_clusters <= 0 || n_clusters > kEmbedMaxClusters) return FLOP_ERR_SHAPE;
    if (!cl) return FLOP_ERR_NULL;
    for (int c = 0; c < n_clusters; ++c) {
        if (cl[c].dim <= 0 || cl[c].dim > kMaxDim || cl[c].id_begin < 0 || cl[c].id_end <= cl[c].id_begin ||
            cl[c].id_end > ((int64_t)1 << 31))
            return FLOP_ERR_SHAPE;
        if (c > 0 && cl[c].id_begin < cl[c - 1].id_end) return FLOP_ERR_SHAPE;   // ascending, disjoint
        if (!cl[c].E || !cl[c].O || !cl[c].z) return FLOP_ERR_NULL;
        if (cl[c].lde < cl[c].dim || cl[c].ldo < d) return FLOP_ERR_STRIDE;
        dims[c] = cl[c].dim;
    }
    return FLOP_OK;
}

// dlog_alpha_k = (sum_i dh_ik g_ik) / z_k^2 * dzda_k: chunked column reduction, then the finish kernel.
int launch_gate_grad(flop_dtype dt, int64_t n, int64_t r, const void* dh, int64_t ldh, const void* g, int64_t ldg,
                     const float* z, const float* dzda, float* dlog_alpha, int accumulate, float* partial,
                     hipStream_t st, const int32_t* r_active = nullptr, flop_gate_grad_pending* pending = nullptr,
                     const int32_t* out_map = nullptr)
{
    // 32-row chunks fill the chip for small n; long inputs use 128-row chunks (more loads in flight per lane)
    const int chunk_rows = (n >= 16384) ? 128 : kColsumChunkRows;
    const int chunks = (int)((n + chunk_rows - 1) / chunk_rows);
    if (chunks > 0) {
        const int es = (int)elem_size(dt);
        const int cols_per_block = 32 * (16 / es);
        const dim3 grid((unsigned)chunks, (unsigned)((r + cols_per_block - 1) / cols_per_block));
        const int vec = aligned16(dh) && aligned16(g) && (ldh * es) % 16 == 0 && (ldg * es) % 16 == 0;
        if (dt == FLOP_BF16)
            hipLaunchKernelGGL(colsum_dot_kernel<2>, grid, dim3(kStreamThreads), 0, st, dh, ldh, g, ldg, (int)n, (int)r,
                               partial, vec, (const int32_t*)nullptr, chunk_rows);
        else
            hipLaunchKernelGGL(colsum_dot_kernel<4>, grid, dim3(kStreamThreads), 0, st, dh, ldh, g, ldg, (int)n, (int)r,
                               partial, vec, (const int32_t*)nullptr, chunk_rows);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    if (pending) {   // the caller finishes several gate vectors in one launch later
        *pending = {partial, z, dzda, dlog_alpha, r_active, r, chunks, accumulate};
        return FLOP_OK;
    }
    hipLaunchKernelGGL(dalpha_finish_kernel, dim3((unsigned)((r + 31) / 32)), dim3(kStreamThreads), 0, st,
                       (const float*)partial, chunks, r, z, dzda, dlog_alpha, accumulate, (const int32_t*)nullptr, chunk_rows,
                       r_active, out_map);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

// r_active (nullable): device int with the number of leading ranks in use (after compaction); r is then
// the capacity of the buffers and sizes the grids.
int fwd_impl(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, const int32_t* r_active, void* g_saved, int64_t ldg, void* y, int64_t ldy,
             void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || r <= 0 || dout <= 0) return FLOP_ERR_SHAPE;
    if (n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (n == 0) return FLOP_OK;
    if (!x || !Q || !P || !z || !g_saved || !y) return FLOP_ERR_NULL;
    if (ldx < d || ldq < d || ldp < r || ldg < r || ldy < dout) return FLOP_ERR_STRIDE;
    if (ld_too_large({ldx, ldq, ldp, ldg, ldy})) return FLOP_ERR_STRIDE;
    if (workspace && ((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    if (!workspace) workspace_bytes = 0;   // the workspace is optional: it only enables k-split launches

    // g = (x Q^T) .* z
    GemmDesc g1 = {x, ldx, true, Q, ldq, true, g_saved, ldg, n, r, d, z};
    g1.ext = r_active; g1.ext_dim = 3;
    int rc = launch_group(dt, &g1, 1, st, nullptr, workspace, workspace_bytes);
    if (rc != FLOP_OK) return rc;
    // y = g P^T
    GemmDesc g2 = {g_saved, ldg, true, P, ldp, true, y, ldy, n, dout, r, nullptr};
    g2.ext = r_active; g2.ext_dim = 2;
    return launch_group(dt, &g2, 1, st, nullptr, workspace, workspace_bytes);
}

// ---- step boundary: gate-gradient finish of the ending step + gates and Eq.(3) of the next one -----------------
// Host-side checks shared by flop_step_boundary and flop_bwd_boundary.
int boundary_check(const flop_gate_grad_pending* items, int count, const flop_boundary_job& j)
{
    if (!valid_hc(j.hc)) return FLOP_ERR_PARAM;
    if (count < 0 || j.n_gates < 0 || j.n_gates > ((int64_t)1 << 40)) return FLOP_ERR_SHAPE;
    if (count > 0 && !items) return FLOP_ERR_NULL;
    if (j.n_gates > 0 && (!j.l0_sum || !j.log_alpha || !j.u || !j.z)) return FLOP_ERR_NULL;
    auto overlap = [](const float* a, int64_t na, const float* b, int64_t nb) {
        return a && b && na > 0 && nb > 0 && (uintptr_t)a < (uintptr_t)(b + nb) && (uintptr_t)b < (uintptr_t)(a + na);
    };
    for (int i = 0; i < count; ++i) {
        const flop_gate_grad_pending& it = items[i];
        if (it.r <= 0 || it.r > kMaxDim || it.chunks < 0) return FLOP_ERR_SHAPE;
        if (!it.z || !it.dzda || !it.dlog_alpha || (it.chunks > 0 && !it.partial)) return FLOP_ERR_NULL;
        const float* read_or_written[3] = {it.z, it.dzda, it.dlog_alpha};
        for (const float* p : read_or_written)
            if (overlap(j.z, j.n_gates, p, it.r) || overlap(j.dzda, j.n_gates, p, it.r) ||
                overlap(j.l0_grad, j.n_gates, p, it.r) || overlap(j.l0_sum, 1, p, it.r))
                return FLOP_ERR_ALIAS;
    }
    return FLOP_OK;
}

// One launch holds the boundary when at most kFinishBatch gate vectors and 4096 new gates are involved.
inline bool boundary_fits(int count, const flop_boundary_job& j)
{
    return count >= 0 && count <= kFinishBatch && j.n_gates >= 0 && j.n_gates <= 4096;
}

void boundary_fill(BoundaryRider& br, const flop_gate_grad_pending* items, int count, const flop_boundary_job& j)
{
    memset(&br, 0, sizeof(br));
    int64_t max_r = 32;
    for (int v = 0; v < count; ++v) {
        const flop_gate_grad_pending& it = items[v];
        br.fb.partial[v] = it.partial; br.fb.z[v] = it.z; br.fb.dzda[v] = it.dzda; br.fb.dlog_alpha[v] = it.dlog_alpha;
        br.fb.r_active[v] = it.r_active; br.fb.r[v] = it.r; br.fb.chunks[v] = it.chunks; br.fb.chunk_rows[v] = 1;
        br.fb.accumulate[v] = it.accumulate;
        if (it.r > max_r) max_r = it.r;
    }
    br.gj = {j.log_alpha, j.u, j.w, j.z, j.dzda, j.l0_grad, j.l0_sum, (int)j.n_gates, j.hc.beta, j.hc.l, j.hc.r,
             j.hc.beta * logf(-j.hc.l / j.hc.r)};
    br.count = count;
    br.bx = (int)((max_r + 31) / 32);
}

// The boundary as launches of its own: one if it fits, else the finish and the gate kernels one after the other.
int boundary_launch(const flop_gate_grad_pending* items, int count, const flop_boundary_job& j, void* stream)
{
    if (j.n_gates == 0) return flop_gate_grad_finish(items, count, stream);   // nothing to sample
    if (count == 0 || !boundary_fits(count, j)) {
        const int rc = flop_gate_grad_finish(items, count, stream);
        if (rc != FLOP_OK) return rc;
        return flop_gate_sample_l0(j.log_alpha, j.u, j.n_gates, j.hc, j.z, j.dzda, j.w, j.l0_sum, j.l0_grad,
                                   j.workspace, j.workspace_bytes, stream);
    }
    BoundaryRider br;
    boundary_fill(br, items, count, j);
    hipLaunchKernelGGL(step_boundary_kernel, dim3((unsigned)br.bx, (unsigned)(count + 1)), dim3(kStreamThreads), 0,
                       (hipStream_t)stream, br.fb, count, br.gj);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int bwd_impl(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* dy, int64_t lddy, const void* x, int64_t ldx,
             const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, const float* dzda, const int32_t* r_active, const void* g_saved, int64_t ldg,
             void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
             float* dlog_alpha, int accumulate,
             void* workspace, size_t workspace_bytes, void* stream, flop_gate_grad_pending* pending = nullptr,
             const flop_boundary_job* boundary = nullptr, flop_weight_grad_pending* weights = nullptr)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || r <= 0 || dout <= 0) return FLOP_ERR_SHAPE;
    if (n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (!Q || !P || !z) return FLOP_ERR_NULL;
    if (n > 0 && (!dy || !x || !g_saved)) return FLOP_ERR_NULL;
    if (dlog_alpha && !dzda) return FLOP_ERR_NULL;
    if (pending && !dlog_alpha) return FLOP_ERR_NULL;
    if (lddy < dout || ldx < d || ldq < d || ldp < r || ldg < r) return FLOP_ERR_STRIDE;
    if ((dx && lddx < d) || (dQ && lddq < d) || (dP && lddp < r)) return FLOP_ERR_STRIDE;
    if (ld_too_large({lddy, ldx, ldq, ldp, ldg, lddx, lddq, lddp})) return FLOP_ERR_STRIDE;
    if (!workspace || workspace_bytes < flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout))
        return FLOP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;

    void* dh = workspace;
    const int64_t ldh = bwd_ldh(r, dt);
    float* partial = (float*)((char*)workspace + bwd_dh_bytes(n, r, dt));
    void* split_ws = (char*)workspace + bwd_dh_bytes(n, r, dt) + bwd_partial_bytes(n, r);
    const size_t split_bytes = bwd_split_bytes(n, d, r, dout);
    const bool need_dh = dx || dQ || dlog_alpha;
    int rc;
    if (weights) {   // dP and dQ are left to flop_weight_grad_finish: this call only records their operands
        *weights = {(int32_t)dt, n, d, r, dout, dy, lddy, g_saved, ldg, dQ ? dh : nullptr, ldh, x, ldx, dP, lddp, dQ, lddq,
                    split_ws, split_bytes};
        dP = nullptr;
        dQ = nullptr;
    }

    // Phase 1: dh = (dy P) .* z and dP = dy^T g.
    GemmDesc ph1[2];
    int c1 = 0;
    // With (at least 4-byte) aligned rows of g the first product also leaves, per tile row, the column
    // sums of dh .* g that the gate gradient needs (no second pass over dh and g).
    int fused_rows = 0;
    if (need_dh && n > 0) {
        ph1[c1] = {dy, lddy, true, P, ldp, false, dh, ldh, n, r, dout, z};
        ph1[c1].ext = r_active; ph1[c1].ext_dim = 3;
        if (dlog_alpha && dt == FLOP_BF16 && ((uintptr_t)g_saved & 3u) == 0 && ldg % 2 == 0) {
            ph1[c1].dot = g_saved; ph1[c1].lddot = ldg; ph1[c1].dot_partial = partial;
        }
        ++c1;
    }
    if (dP) {
        ph1[c1] = {dy, lddy, false, g_saved, ldg, false, dP, lddp, dout, r, n, nullptr};
        ph1[c1].ext = r_active; ph1[c1].ext_dim = 3;
        ++c1;
    }
    if (c1) { rc = launch_group(dt, ph1, c1, st, &fused_rows, split_ws, split_bytes); if (rc != FLOP_OK) return rc; }
    if (!(need_dh && n > 0 && ph1[0].dot_partial)) fused_rows = 0;

    // Phase 2: dQ = dh^T x and dx = dh Q.
    GemmDesc ph2[2];
    int c2 = 0;
    if (dQ) {
        ph2[c2] = {dh, ldh, false, x, ldx, false, dQ, lddq, r, d, n, nullptr};
        ph2[c2].ext = r_active; ph2[c2].ext_dim = 1;
        ++c2;
    }
    if (dx && n > 0) {
        ph2[c2] = {dh, ldh, true, Q, ldq, false, dx, lddx, n, d, r, nullptr};
        ph2[c2].ext = r_active; ph2[c2].ext_dim = 2;
        ++c2;
    }
    // With a step boundary to serve (flop_bwd_boundary) and this layer's column sums already complete, the
    // boundary work - this layer's gate gradient included - rides on the launch of phase 2.
    flop_gate_grad_pending all_items[kFinishBatch + 1];
    int n_items = 0;
    bool carried = false;
    if (boundary) {
        for (int i = 0; i < boundary->count && i < kFinishBatch; ++i) all_items[n_items++] = boundary->items[i];
        const bool own_ready = !dlog_alpha || fused_rows != 0;
        if (c2 && own_ready && boundary->count + (dlog_alpha ? 1 : 0) <= kFinishBatch && boundary_fits(boundary->count, *boundary)) {
            if (dlog_alpha)
                all_items[n_items++] = {partial, z, dzda, dlog_alpha, r_active, r, (int)((n + fused_rows - 1) / fused_rows), accumulate};
            BoundaryRider br;
            boundary_fill(br, all_items, n_items, *boundary);
            rc = launch_group(dt, ph2, c2, st, nullptr, split_ws, split_bytes, &br, &carried);
            if (rc != FLOP_OK) return rc;
            if (carried) return FLOP_OK;
            if (dlog_alpha) --n_items;   // not carried: this layer's item is written again below
            c2 = 0;                      // phase 2 has been launched
        }
    }
    if (c2) { rc = launch_group(dt, ph2, c2, st, nullptr, split_ws, split_bytes); if (rc != FLOP_OK) return rc; }

    flop_gate_grad_pending own;
    if (boundary && dlog_alpha) pending = &own;
    // Gate gradient: column reduction of dh .* g, then dlog_alpha = (sum / z^2) * dzda.
    if (dlog_alpha && fused_rows) {
        const int chunks = (int)((n + fused_rows - 1) / fused_rows);
        if (pending) {
            *pending = {partial, z, dzda, dlog_alpha, r_active, r, chunks, accumulate};
        } else {
            hipLaunchKernelGGL(dalpha_finish_kernel, dim3((unsigned)((r + 31) / 32)), dim3(kStreamThreads), 0, st,
                               (const float*)partial, chunks, r, z, dzda, dlog_alpha,
                               accumulate, (const int32_t*)nullptr, fused_rows, r_active, (const int32_t*)nullptr);
            if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
        }
    } else if (dlog_alpha) {
        rc = launch_gate_grad(dt, n, r, dh, ldh, g_saved, ldg, z, dzda, dlog_alpha, accumulate, partial, st, r_active, pending);
        if (rc != FLOP_OK) return rc;
    }
    if (boundary) {   // the boundary did not ride: launches of its own, in as few as the counts allow
        if (boundary->count > kFinishBatch) {   // the caller's list is longer than the local copy
            rc = flop_gate_grad_finish(boundary->items, boundary->count, stream);
            if (rc != FLOP_OK) return rc;
            n_items = 0;
        }
        if (dlog_alpha) all_items[n_items++] = own;
        return boundary_launch(all_items, n_items, *boundary, stream);
    }
    return FLOP_OK;
}

// ------------------------------------------------------------------------
// Scratch of flop_bwd_static: one array in device memory per GPU, part of the code object.  In host code the
// array's name only stands for the symbol; its device address is looked up once per device and kept.
// ------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[FLOP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct ScratchTable {
    std::mutex mu;
    void* ptr[kMaxDevices] = {};
} g_scratch;

// Device address of `scratch` on the current device, or nullptr if the lookup fails.
void* scratch_ptr()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch.mu);
    if (!g_scratch.ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch.ptr[dev] = p;
    }
    return g_scratch.ptr[dev];
}

inline int l0_blocks(int64_t n)
{
    int64_t b = (n + (int64_t)kStreamThreads * 16 - 1) / ((int64_t)kStreamThreads * 16);
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;
    return (int)b;
}

}  // namespace

extern "C" {

const char* flop_status_string(int status)
{
    switch (status) {
        case FLOP_OK: return "ok";
        case FLOP_ERR_NULL: return "required pointer is NULL";
        case FLOP_ERR_SHAPE: return "invalid size";
        case FLOP_ERR_STRIDE: return "leading dimension smaller than row length";
        case FLOP_ERR_DTYPE: return "unknown dtype or mode";
        case FLOP_ERR_PARAM: return "hard-concrete constants need l < 0, r > 1, beta > 0";
        case FLOP_ERR_WORKSPACE: return "workspace missing or too small";
        case FLOP_ERR_ALIGN: return "workspace not 256-byte aligned";
        case FLOP_ERR_HIP: return "HIP launch failed";
        case FLOP_ERR_ALIAS: return "an output overlaps an input of the same launch";
        case FLOP_ERR_SCRATCH: return "problem needs more scratch than the static device array holds (FLOP_STATIC_SCRATCH_BYTES)";
        default: return "unknown status";
    }
}

size_t flop_workspace_bytes(int op, flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout)
{
    if (!valid_dtype(dt) || n < 0 || r < 0) return 0;
    switch (op) {
        case FLOP_OP_FWD:
            return (dt == FLOP_BF16 && d > 0 && dout > 0) ? fwd_split_bytes(n, d, r, dout) : 0;
        case FLOP_OP_BWD:
            return bwd_dh_bytes(n, r, dt) + bwd_partial_bytes(n, r) +
                   ((dt == FLOP_BF16 && d > 0 && dout > 0) ? bwd_split_bytes(n, d, r, dout) : 0);
        case FLOP_OP_EXPECTED_L0:
            return 2048 * sizeof(double);
        case FLOP_OP_GATE_GRAD:
            return (size_t)round_up(((n + kColsumChunkRows - 1) / kColsumChunkRows) * r * 4, 256);
        case FLOP_OP_EMBED_FWD:   /* n tokens, r = sum of cluster dimensions: bytes of `saved` */
            return embed_saved_bound(dt, n, r);
        case FLOP_OP_EMBED_BWD:
            return embed_ws_bound(dt, n, d, r);
        default:
            return 0;
    }
}

int flop_gate_sample(const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                     flop_gate_mode mode, float* z, float* dzda, void* stream)
{
    if (mode != FLOP_GATE_TRAIN && mode != FLOP_GATE_DETERMINISTIC) return FLOP_ERR_DTYPE;
    if (!valid_hc(hc)) return FLOP_ERR_PARAM;
    if (n_gates < 0 || n_gates > ((int64_t)1 << 40)) return FLOP_ERR_SHAPE;
    if (n_gates == 0) return FLOP_OK;
    if (!log_alpha || !z || (mode == FLOP_GATE_TRAIN && !u)) return FLOP_ERR_NULL;
    const bool vec = aligned16(log_alpha) && aligned16(z) && (mode != FLOP_GATE_TRAIN || aligned16(u)) &&
                     (!dzda || aligned16(dzda));
    hipStream_t st = (hipStream_t)stream;
    if (vec) {
        int64_t blocks = (n_gates + kStreamThreads * 4 - 1) / (kStreamThreads * 4);
        if (blocks > 4096) blocks = 4096;   // 16 blocks per CU, grid-stride beyond that
        hipLaunchKernelGGL(gate_sample_kernel<4>, dim3((unsigned)blocks), dim3(kStreamThreads), 0, st,
                           log_alpha, u, n_gates, hc.beta, hc.l, hc.r, (int)mode, z, dzda);
    } else {
        int64_t blocks = (n_gates + kStreamThreads - 1) / kStreamThreads;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(gate_sample_kernel<1>, dim3((unsigned)blocks), dim3(kStreamThreads), 0, st,
                           log_alpha, u, n_gates, hc.beta, hc.l, hc.r, (int)mode, z, dzda);
    }
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_fwd(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, void* g_saved, int64_t ldg, void* y, int64_t ldy,
             void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_impl(dt, n, d, r, dout, x, ldx, Q, ldq, P, ldp, z, nullptr, g_saved, ldg, y, ldy, workspace,
                    workspace_bytes, stream);
}

int flop_fwd_sampling(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const flop_boundary_job* job, int64_t gate_offset, void* g_saved, int64_t ldg, void* y, int64_t ldy,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    if (!job) return FLOP_ERR_NULL;
    if (job->count != 0 || gate_offset < 0 || r <= 0 || gate_offset + r > job->n_gates) return FLOP_ERR_SHAPE;
    int rc = boundary_check(nullptr, 0, *job);
    if (rc != FLOP_OK) return rc;
    if (!job->dzda) return FLOP_ERR_NULL;
    // the checks of flop_fwd, before anything is launched
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || dout <= 0 || n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (n > 0 && (!x || !Q || !P || !g_saved || !y)) return FLOP_ERR_NULL;
    if (ldx < d || ldq < d || ldp < r || ldg < r || ldy < dout) return FLOP_ERR_STRIDE;
    if (ld_too_large({ldx, ldq, ldp, ldg, ldy})) return FLOP_ERR_STRIDE;
    if (workspace && ((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    GemmDesc g1 = {x, ldx, true, Q, ldq, true, g_saved, ldg, n, r, d, nullptr};
    if (n > 0 && boundary_fits(0, *job) && gate_fusable(dt, g1)) {
        // g = (x Q^T) .* z with z computed in the epilogue; extra workgroups write every gate of the job and Eq.(3)
        g1.gate_alpha = job->log_alpha + gate_offset; g1.gate_u = job->u + gate_offset;
        g1.gate_beta = job->hc.beta; g1.gate_l = job->hc.l; g1.gate_r = job->hc.r;
        BoundaryRider br;
        boundary_fill(br, nullptr, 0, *job);
        bool carried = false;
        rc = launch_group(dt, &g1, 1, st, nullptr, nullptr, 0, &br, &carried);
        if (rc != FLOP_OK) return rc;
        if (!carried) return FLOP_ERR_HIP;
        GemmDesc g2 = {g_saved, ldg, true, P, ldp, true, y, ldy, n, dout, r, nullptr};
        return launch_group(dt, &g2, 1, st, nullptr, workspace, workspace ? workspace_bytes : 0);
    }
    rc = boundary_launch(nullptr, 0, *job, stream);
    if (rc != FLOP_OK) return rc;
    return fwd_impl(dt, n, d, r, dout, x, ldx, Q, ldq, P, ldp, job->z + gate_offset, nullptr, g_saved, ldg, y, ldy,
                    workspace, workspace_bytes, stream);
}

int flop_fwd_active(flop_dtype dt, int64_t n, int64_t d, int64_t r_cap, int64_t dout,
                    const void* x, int64_t ldx, const void* Qc, int64_t ldqc, const void* Pc, int64_t ldpc,
                    const float* zc, const int32_t* r_active, void* g_saved, int64_t ldg, void* y, int64_t ldy,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!r_active) return FLOP_ERR_NULL;
    return fwd_impl(dt, n, d, r_cap, dout, x, ldx, Qc, ldqc, Pc, ldpc, zc, r_active, g_saved, ldg, y, ldy, workspace,
                    workspace_bytes, stream);
}

int flop_bwd(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* dy, int64_t lddy, const void* x, int64_t ldx,
             const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, const float* dzda, const void* g_saved, int64_t ldg,
             void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
             float* dlog_alpha, int accumulate,
             void* workspace, size_t workspace_bytes, void* stream)
{
    return bwd_impl(dt, n, d, r, dout, dy, lddy, x, ldx, Q, ldq, P, ldp, z, dzda, nullptr, g_saved, ldg, dx, lddx,
                    dQ, lddq, dP, lddp, dlog_alpha, accumulate, workspace, workspace_bytes, stream);
}

int flop_bwd_static(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                    const void* dy, int64_t lddy, const void* x, int64_t ldx,
                    const void* Q, int64_t ldq, const void* P, int64_t ldp,
                    const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                    void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                    float* dlog_alpha, int accumulate, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || r <= 0 || dout <= 0 || n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim)
        return FLOP_ERR_SHAPE;
    if (flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout) > FLOP_STATIC_SCRATCH_BYTES) return FLOP_ERR_SCRATCH;
    void* ws = scratch_ptr();
    if (!ws) return FLOP_ERR_HIP;
    return bwd_impl(dt, n, d, r, dout, dy, lddy, x, ldx, Q, ldq, P, ldp, z, dzda, nullptr, g_saved, ldg, dx, lddx,
                    dQ, lddq, dP, lddp, dlog_alpha, accumulate, ws, FLOP_STATIC_SCRATCH_BYTES, stream);
}

int flop_bwd_deferred(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* dy, int64_t lddy, const void* x, int64_t ldx,
                      const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                      void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                      float* dlog_alpha, int accumulate,
                      void* workspace, size_t workspace_bytes, void* stream,
                      flop_gate_grad_pending* pending)
{
    if (!pending) return FLOP_ERR_NULL;
    return bwd_impl(dt, n, d, r, dout, dy, lddy, x, ldx, Q, ldq, P, ldp, z, dzda, nullptr, g_saved, ldg, dx, lddx,
                    dQ, lddq, dP, lddp, dlog_alpha, accumulate, workspace, workspace_bytes, stream, pending);
}

int flop_bwd_defer_weights(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                           const void* dy, int64_t lddy, const void* x, int64_t ldx,
                           const void* Q, int64_t ldq, const void* P, int64_t ldp,
                           const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                           void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                           float* dlog_alpha, int accumulate,
                           void* workspace, size_t workspace_bytes, void* stream,
                           flop_gate_grad_pending* pending, flop_weight_grad_pending* weights)
{
    if (!weights || (dlog_alpha && !pending)) return FLOP_ERR_NULL;
    return bwd_impl(dt, n, d, r, dout, dy, lddy, x, ldx, Q, ldq, P, ldp, z, dzda, nullptr, g_saved, ldg, dx, lddx,
                    dQ, lddq, dP, lddp, dlog_alpha, accumulate, workspace, workspace_bytes, stream,
                    dlog_alpha ? pending : nullptr, nullptr, weights);
}

int flop_weight_grad_finish(const flop_weight_grad_pending* items, int32_t count, void* stream)
{
    if (count < 0) return FLOP_ERR_SHAPE;
    if (count == 0) return FLOP_OK;
    if (!items) return FLOP_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const flop_weight_grad_pending& it = items[i];
        if (!valid_dtype(it.dtype)) return FLOP_ERR_DTYPE;
        if (it.n < 0 || it.d <= 0 || it.r <= 0 || it.dout <= 0) return FLOP_ERR_SHAPE;
        if (it.n > kMaxDim || it.d > kMaxDim || it.r > kMaxDim || it.dout > kMaxDim) return FLOP_ERR_SHAPE;
        if (it.dP && it.n > 0 && (!it.dy || !it.g)) return FLOP_ERR_NULL;
        if (it.dQ && it.n > 0 && (!it.dh || !it.x)) return FLOP_ERR_NULL;
        if (it.dP && (it.lddy < it.dout || it.ldg < it.r || it.lddp < it.r)) return FLOP_ERR_STRIDE;
        if (it.dQ && (it.ldh < it.r || it.ldx < it.d || it.lddq < it.d)) return FLOP_ERR_STRIDE;
        if (ld_too_large({it.lddy, it.ldg, it.ldh, it.ldx, it.lddp, it.lddq})) return FLOP_ERR_STRIDE;
    }
    hipStream_t st = (hipStream_t)stream;
    // Class of a product for sharing a launch: 0 = none (launched with its layer only), 1 = float32 (generic
    // kernel), 16 / 4 = bfloat16 on the transfer kernel, unsplit, with transfers of that many bytes.  A launch
    // runs at the narrowest width of its members, so the classes are kept apart.
    auto share_class = [](flop_dtype dt, const GemmDesc& g) {
        if (g.K <= 0) return 0;
        if (dt != FLOP_BF16) return 1;
        int min_split = 1;
        const int w = dma_width(g, &min_split);
        return min_split == 1 ? w : 0;
    };
    GemmDesc batch[kMaxGroup];
    int nb = 0, batch_layers = 0, batch_dt = FLOP_BF16, batch_cls = 0;
    const flop_weight_grad_pending* batch_first = nullptr;
    int rc = FLOP_OK;
    auto flush = [&]() {
        if (nb == 0) return (int)FLOP_OK;
        // a launch that serves a single layer may cut its products along k into that layer's scratch
        const bool one = batch_layers == 1;
        const int rcl = launch_group((flop_dtype)batch_dt, batch, nb, st, nullptr, one ? batch_first->split_ws : nullptr,
                                     one ? batch_first->split_bytes : 0);
        nb = 0;
        batch_layers = 0;
        return rcl;
    };
    for (int i = 0; i < count; ++i) {
        const flop_weight_grad_pending& it = items[i];
        GemmDesc pr[2];
        int c = 0;
        if (it.dP) pr[c++] = {it.dy, it.lddy, false, it.g, it.ldg, false, it.dP, it.lddp, it.dout, it.r, it.n, nullptr};
        if (it.dQ) pr[c++] = {it.dh, it.ldh, false, it.x, it.ldx, false, it.dQ, it.lddq, it.r, it.d, it.n, nullptr};
        if (c == 0) continue;
        int cls = share_class((flop_dtype)it.dtype, pr[0]);
        if (c == 2) { const int c1 = share_class((flop_dtype)it.dtype, pr[1]); cls = c1 < cls ? c1 : cls; }
        if (cls == 0) {   // on its own, with everything launch_group can fall back to
            if ((rc = flush()) != FLOP_OK) return rc;
            rc = launch_group((flop_dtype)it.dtype, pr, c, st, nullptr, it.split_ws, it.split_bytes);
            if (rc != FLOP_OK) return rc;
            continue;
        }
        if (nb + c > kMaxGroup || (nb && (batch_dt != it.dtype || batch_cls != cls)))
            if ((rc = flush()) != FLOP_OK) return rc;
        if (nb == 0) { batch_first = &it; batch_dt = it.dtype; batch_cls = cls; }
        for (int q = 0; q < c; ++q) { batch[nb] = pr[q]; batch[nb++].few_xcds = true; }
        ++batch_layers;
    }
    return flush();
}

int flop_gate_grad_finish(const flop_gate_grad_pending* items, int32_t count, void* stream)
{
    if (count < 0) return FLOP_ERR_SHAPE;
    if (count == 0) return FLOP_OK;
    if (!items) return FLOP_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        if (items[i].r <= 0 || items[i].r > kMaxDim || items[i].chunks < 0) return FLOP_ERR_SHAPE;
        if (!items[i].z || !items[i].dzda || !items[i].dlog_alpha || (items[i].chunks > 0 && !items[i].partial)) return FLOP_ERR_NULL;
    }
    for (int i0 = 0; i0 < count; i0 += kFinishBatch) {
        FinishBatch fb;
        memset(&fb, 0, sizeof(fb));
        int64_t max_r = 0;
        const int m = count - i0 < kFinishBatch ? count - i0 : kFinishBatch;
        for (int v = 0; v < m; ++v) {
            const flop_gate_grad_pending& it = items[i0 + v];
            fb.partial[v] = it.partial; fb.z[v] = it.z; fb.dzda[v] = it.dzda; fb.dlog_alpha[v] = it.dlog_alpha;
            fb.r_active[v] = it.r_active; fb.r[v] = it.r; fb.chunks[v] = it.chunks; fb.chunk_rows[v] = 1;
            fb.accumulate[v] = it.accumulate;
            if (it.r > max_r) max_r = it.r;
        }
        hipLaunchKernelGGL(dalpha_finish_batch_kernel, dim3((unsigned)((max_r + 31) / 32), (unsigned)m), dim3(kStreamThreads), 0,
                           (hipStream_t)stream, fb);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    return FLOP_OK;
}

int flop_bwd_active(flop_dtype dt, int64_t n, int64_t d, int64_t r_cap, int64_t dout,
                    const void* dy, int64_t lddy, const void* x, int64_t ldx,
                    const void* Qc, int64_t ldqc, const void* Pc, int64_t ldpc,
                    const float* zc, const float* dzda_c, const int32_t* r_active, const void* g_saved, int64_t ldg,
                    void* dx, int64_t lddx, void* dQc, int64_t lddqc, void* dPc, int64_t lddpc,
                    float* dlog_alpha_c, int accumulate,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    if (!r_active) return FLOP_ERR_NULL;
    return bwd_impl(dt, n, d, r_cap, dout, dy, lddy, x, ldx, Qc, ldqc, Pc, ldpc, zc, dzda_c, r_active, g_saved, ldg,
                    dx, lddx, dQc, lddqc, dPc, lddpc, dlog_alpha_c, accumulate, workspace, workspace_bytes, stream);
}

// ---- active ranks read in place (flop.h: flop_fwd_active_indexed / flop_bwd_active_indexed) -------------------
int flop_fwd_active_indexed(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                            const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* Pt, int64_t ldpt,
                            const float* zc, const int32_t* idx, const int32_t* r_active,
                            void* g_active, int64_t ldg, void* y, int64_t ldy, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || r <= 0 || dout <= 0) return FLOP_ERR_SHAPE;
    if (n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (n == 0) return FLOP_OK;
    if (!x || !Q || !Pt || !zc || !idx || !r_active || !g_active || !y) return FLOP_ERR_NULL;
    if (ldx < d || ldq < d || ldpt < dout || ldg < r || ldy < dout) return FLOP_ERR_STRIDE;
    if (ld_too_large({ldx, ldq, ldpt, ldg, ldy})) return FLOP_ERR_STRIDE;
    hipStream_t st = (hipStream_t)stream;
    // g = (x Q[idx]^T) .* zc: the rows of Q are gathered
    GemmDesc g1 = {x, ldx, true, Q, ldq, true, g_active, ldg, n, r, d, zc};
    g1.ext = r_active; g1.ext_dim = 3; g1.b_map = idx; g1.b_map_rows = r;
    int rc = launch_group(dt, &g1, 1, st);
    if (rc != FLOP_OK) return rc;
    // y = g Pt[idx]: the contraction runs down the gathered rows of Pt
    GemmDesc g2 = {g_active, ldg, true, Pt, ldpt, false, y, ldy, n, dout, r, nullptr};
    g2.ext = r_active; g2.ext_dim = 2; g2.b_map = idx; g2.b_map_rows = r;
    return launch_group(dt, &g2, 1, st);
}

int flop_bwd_active_indexed(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                            const void* dy, int64_t lddy, const void* x, int64_t ldx,
                            const void* Q, int64_t ldq, const void* Pt, int64_t ldpt,
                            const float* zc, const float* dzda_c, const int32_t* idx, const int32_t* r_active,
                            const void* g_active, int64_t ldg,
                            void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dPt, int64_t lddpt,
                            float* dlog_alpha, int accumulate,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || d <= 0 || r <= 0 || dout <= 0) return FLOP_ERR_SHAPE;
    if (n > kMaxDim || d > kMaxDim || r > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (!Q || !Pt || !zc || !idx || !r_active) return FLOP_ERR_NULL;
    if (n > 0 && (!dy || !x || !g_active)) return FLOP_ERR_NULL;
    if (dlog_alpha && !dzda_c) return FLOP_ERR_NULL;
    if (lddy < dout || ldx < d || ldq < d || ldpt < dout || ldg < r) return FLOP_ERR_STRIDE;
    if ((dx && lddx < d) || (dQ && lddq < d) || (dPt && lddpt < dout)) return FLOP_ERR_STRIDE;
    if (ld_too_large({lddy, ldx, ldq, ldpt, ldg, lddx, lddq, lddpt})) return FLOP_ERR_STRIDE;
    if (!workspace || workspace_bytes < flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout)) return FLOP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int es = (int)elem_size(dt);

    // closed components: exact zeros in their rows of dQ and dPt and (unless added to) entries of dlog_alpha; the
    // rows of the open ones are written by the products below
    if (dQ || dPt || (dlog_alpha && !accumulate)) {
        hipLaunchKernelGGL(zero_closed_rows_kernel, dim3((unsigned)r), dim3(kStreamThreads), 0, st, idx, r_active, (int)r,
                           dQ, lddq, (int)d, dPt, lddpt, (int)dout, es, (dlog_alpha && !accumulate) ? dlog_alpha : (float*)nullptr);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    if (n == 0) return FLOP_OK;

    void* dh = workspace;
    const int64_t ldh = bwd_ldh(r, dt);
    float* partial = (float*)((char*)workspace + bwd_dh_bytes(n, r, dt));
    const bool need_dh = dx || dQ || dlog_alpha;
    int rc;
    int fused_rows = 0;
    // dh = (dy Pt[idx]^T) .* zc (rows of Pt gathered), with the column sums of dh .* g where the kernel can
    if (need_dh) {
        GemmDesc p1 = {dy, lddy, true, Pt, ldpt, true, dh, ldh, n, r, dout, zc};
        p1.ext = r_active; p1.ext_dim = 3; p1.b_map = idx; p1.b_map_rows = r;
        if (dlog_alpha && dt == FLOP_BF16 && ((uintptr_t)g_active & 3u) == 0 && ldg % 2 == 0) {
            p1.dot = g_active; p1.lddot = ldg; p1.dot_partial = partial;
        }
        rc = launch_group(dt, &p1, 1, st, &fused_rows);
        if (rc != FLOP_OK) return rc;
        if (!p1.dot_partial) fused_rows = 0;
    }
    // dPt[idx] = g^T dy, dQ[idx] = dh^T x (rows scattered by the index list), dx = dh Q[idx] (contraction down
    // the gathered rows of Q): one launch
    GemmDesc p2[3];
    int c2 = 0;
    if (dPt) {
        p2[c2] = {g_active, ldg, false, dy, lddy, false, dPt, lddpt, r, dout, n, nullptr};
        p2[c2].ext = r_active; p2[c2].ext_dim = 1; p2[c2].c_rowmap = idx;
        ++c2;
    }
    if (dQ) {
        p2[c2] = {dh, ldh, false, x, ldx, false, dQ, lddq, r, d, n, nullptr};
        p2[c2].ext = r_active; p2[c2].ext_dim = 1; p2[c2].c_rowmap = idx;
        ++c2;
    }
    if (dx) {
        p2[c2] = {dh, ldh, true, Q, ldq, false, dx, lddx, n, d, r, nullptr};
        p2[c2].ext = r_active; p2[c2].ext_dim = 2; p2[c2].b_map = idx; p2[c2].b_map_rows = r;
        ++c2;
    }
    if (c2) { rc = launch_group(dt, p2, c2, st); if (rc != FLOP_OK) return rc; }

    if (dlog_alpha && fused_rows) {
        const int chunks = (int)((n + fused_rows - 1) / fused_rows);
        hipLaunchKernelGGL(dalpha_finish_kernel, dim3((unsigned)((r + 31) / 32)), dim3(kStreamThreads), 0, st,
                           (const float*)partial, chunks, r, zc, dzda_c, dlog_alpha, accumulate, (const int32_t*)nullptr,
                           fused_rows, r_active, idx);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    } else if (dlog_alpha) {
        rc = launch_gate_grad(dt, n, r, dh, ldh, g_active, ldg, zc, dzda_c, dlog_alpha, accumulate, partial, st, r_active,
                              nullptr, idx);
        if (rc != FLOP_OK) return rc;
    }
    return FLOP_OK;
}

int flop_gather_gates(const float* src, const int32_t* idx, const int32_t* r_active, int64_t r,
                      float* dst, void* stream)
{
    if (r < 0 || r > kMaxDim) return FLOP_ERR_SHAPE;
    if (r == 0) return FLOP_OK;
    if (!src || !idx || !r_active || !dst) return FLOP_ERR_NULL;
    const int blocks = (int)((r + kStreamThreads - 1) / kStreamThreads);
    hipLaunchKernelGGL(gather_gates_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(kStreamThreads), 0,
                       (hipStream_t)stream, src, idx, r_active, dst);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_expand_grads(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                      const int32_t* r_active, const int32_t* idx,
                      const void* dQc, int64_t lddqc, const void* dPc, int64_t lddpc, const float* dlog_alpha_c,
                      void* dQ, int64_t lddq, void* dP, int64_t lddp, float* dlog_alpha, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (r < 0 || d < 0 || dout < 0 || r > kMaxDim || d > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (r == 0) return FLOP_OK;
    if (!r_active || !idx) return FLOP_ERR_NULL;
    if ((dQ && (!dQc || d <= 0)) || (dP && (!dPc || dout <= 0)) || (dlog_alpha && !dlog_alpha_c)) return FLOP_ERR_NULL;
    if ((dQ && (lddq < d || lddqc < d)) || (dP && (lddp < r || lddpc < r))) return FLOP_ERR_STRIDE;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = elem_size(dt);
    const int vec = dQ && aligned16(dQ) && aligned16(dQc) && (lddq * es) % 16 == 0 && (lddqc * es) % 16 == 0;
    const int row_blocks = (dQ || dlog_alpha) ? (int)r : 0;
    // column scatter: 0 = slots by binary search, 1 = slot table in LDS, 2 = slot table and staged rows in LDS
    // with 16-byte accesses (16-byte aligned rows, everything within 64 KB of LDS)
    int use_lds = r <= kExpandMaxLdsRanks;
    size_t lds = (dP && use_lds) ? (size_t)r * sizeof(int32_t) : 0;
    const size_t lds_vec = (size_t)round_up(r, 4) * sizeof(int32_t) + (size_t)kExpandVecRows * (size_t)round_up(r * (int64_t)es, 16);
    if (dP && use_lds && aligned16(dP) && aligned16(dPc) && (lddp * es) % 16 == 0 && (lddpc * es) % 16 == 0 && lds_vec <= 65536) {
        use_lds = 2;
        lds = lds_vec;
    }
    const int rows_per_block = use_lds == 2 ? kExpandVecRows : kExpandRows;
    const int col_blocks = dP ? (int)((dout + rows_per_block - 1) / rows_per_block) : 0;
    if (row_blocks + col_blocks == 0) return FLOP_OK;
    const dim3 grid((unsigned)(row_blocks + col_blocks));
    if (dt == FLOP_BF16)
        hipLaunchKernelGGL(expand_grads_kernel<2>, grid, dim3(kStreamThreads), lds, st, r_active, idx, (int)r, dQc, lddqc,
                           dlog_alpha_c, (int)d, dQ, lddq, dlog_alpha, vec, row_blocks, dPc, lddpc, (int)dout, dP, lddp, use_lds);
    else
        hipLaunchKernelGGL(expand_grads_kernel<4>, grid, dim3(kStreamThreads), lds, st, r_active, idx, (int)r, dQc, lddqc,
                           dlog_alpha_c, (int)d, dQ, lddq, dlog_alpha, vec, row_blocks, dPc, lddpc, (int)dout, dP, lddp, use_lds);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_topk_mask(const float* log_alpha, int64_t n_gates, int64_t keep, const float* keep_device,
                   flop_hc hc, float* z, int32_t* kept, void* stream)
{
    if (!valid_hc(hc)) return FLOP_ERR_PARAM;
    if (n_gates < 0 || n_gates > kMaxDim) return FLOP_ERR_SHAPE;
    if (n_gates > 0 && (!log_alpha || !z)) return FLOP_ERR_NULL;
    const float shift = hc.beta * logf(-hc.l / hc.r);
    hipLaunchKernelGGL(topk_mask_kernel, dim3(1), dim3(kSelectThreads), 0, (hipStream_t)stream,
                       log_alpha, n_gates, keep, keep_device, shift, z, kept);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_lagrangian(const float* size_sum, const float* size_grad, int64_t n_gates, float scale, float t,
                    const float* lambda, float* dlog_alpha, int accumulate, float* out, void* stream)
{
    if (n_gates < 0 || n_gates > ((int64_t)1 << 40)) return FLOP_ERR_SHAPE;
    if (!size_sum || !lambda) return FLOP_ERR_NULL;
    if (dlog_alpha && n_gates > 0 && !size_grad) return FLOP_ERR_NULL;
    if (!dlog_alpha && !out) return FLOP_OK;
    int64_t blocks = (n_gates + kStreamThreads - 1) / kStreamThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(lagrangian_kernel, dim3((unsigned)blocks), dim3(kStreamThreads), 0, (hipStream_t)stream,
                       size_sum, lambda, scale, t, size_grad, n_gates, n_gates > 0 ? dlog_alpha : nullptr, accumulate, out);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_gate_grad(flop_dtype dt, int64_t n, int64_t r, const void* dh, int64_t ldh, const void* g, int64_t ldg,
                   const float* z, const float* dzda, float* dlog_alpha, int accumulate,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (n < 0 || r <= 0 || n > kMaxDim || r > kMaxDim) return FLOP_ERR_SHAPE;
    if (!z || !dzda || !dlog_alpha || (n > 0 && (!dh || !g))) return FLOP_ERR_NULL;
    if (ldh < r || ldg < r) return FLOP_ERR_STRIDE;
    if (!workspace || workspace_bytes < flop_workspace_bytes(FLOP_OP_GATE_GRAD, dt, n, 0, r, 0)) return FLOP_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    return launch_gate_grad(dt, n, r, dh, ldh, g, ldg, z, dzda, dlog_alpha, accumulate, (float*)workspace,
                            (hipStream_t)stream);
}

int flop_expected_l0(const float* log_alpha, const float* w, int64_t n_gates, flop_hc hc,
                     float* out_sum, float* grad,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_hc(hc)) return FLOP_ERR_PARAM;
    if (n_gates < 0 || n_gates > ((int64_t)1 << 40)) return FLOP_ERR_SHAPE;
    if (!out_sum || (n_gates > 0 && !log_alpha)) return FLOP_ERR_NULL;
    const int blocks = l0_blocks(n_gates);
    if (blocks > 1) {
        if (!workspace || workspace_bytes < flop_workspace_bytes(FLOP_OP_EXPECTED_L0, FLOP_F32, n_gates, 0, 0, 0))
            return FLOP_ERR_WORKSPACE;
        if (((uintptr_t)workspace & 255u) != 0) return FLOP_ERR_ALIGN;
    }
    hipStream_t st = (hipStream_t)stream;
    const float shift = hc.beta * logf(-hc.l / hc.r);
    const bool vec = aligned16(log_alpha) && (!w || aligned16(w)) && (!grad || aligned16(grad));
    if (vec)
        hipLaunchKernelGGL(expected_l0_kernel<4>, dim3(blocks), dim3(kStreamThreads), 0, st,
                           log_alpha, w, n_gates, shift, grad, (double*)workspace, out_sum);
    else
        hipLaunchKernelGGL(expected_l0_kernel<1>, dim3(blocks), dim3(kStreamThreads), 0, st,
                           log_alpha, w, n_gates, shift, grad, (double*)workspace, out_sum);
    if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    if (blocks > 1) {
        hipLaunchKernelGGL(expected_l0_finish_kernel, dim3(1), dim3(kStreamThreads), 0, st,
                           (const double*)workspace, blocks, out_sum);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    return FLOP_OK;
}

// Compaction, optionally preceded by the gate sampling of a training step (log_alpha != NULL).
static int compact_impl(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                        const float* z, const void* Q, int64_t ldq, const void* P, int64_t ldp,
                        int absorb_z_into_Q, int32_t* r_out, int32_t* idx,
                        void* Qc, int64_t ldqc, void* Pc, int64_t ldpc, float* zc,
                        const float* log_alpha, const float* u, flop_hc hc, float* z_out, float* dzda_out, float* dzc,
                        hipStream_t st)
{
    if (!valid_dtype(dt)) return FLOP_ERR_DTYPE;
    if (r < 0 || d < 0 || dout < 0 || r > kMaxDim || d > kMaxDim || dout > kMaxDim) return FLOP_ERR_SHAPE;
    if (!r_out) return FLOP_ERR_NULL;
    if (r > 0 && ((!z && !log_alpha) || !idx)) return FLOP_ERR_NULL;
    if (Qc && (!Q || d <= 0)) return FLOP_ERR_NULL;
    if (Pc && (!P || dout <= 0)) return FLOP_ERR_NULL;
    if (Qc && (ldq < d || ldqc < d)) return FLOP_ERR_STRIDE;
    if (Pc && (ldp < r || ldpc < r)) return FLOP_ERR_STRIDE;

    hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, z, (int)r, r_out, idx, zc,
                       log_alpha, u, hc.beta, hc.l, hc.r, z_out, dzda_out, dzc);
    if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    if (r == 0) return FLOP_OK;
    const float* zz = log_alpha ? z_out : z;   // gate values for the optional absorption

    const size_t es = elem_size(dt);
    const bool vec_q = Qc && aligned16(Q) && aligned16(Qc) && (ldq * es) % 16 == 0 && (ldqc * es) % 16 == 0;
    const int vec_p = Pc && aligned16(P) && (ldp * es) % 16 == 0;
    const dim3 block(kStreamThreads);
    if (Qc && Pc) {   // both gathers in one launch
        const dim3 grid((unsigned)(r + dout));
        if (dt == FLOP_BF16) {
            if (vec_q) hipLaunchKernelGGL((compact_gather_kernel<uint16_t, 16>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc, (const uint16_t*)P, ldp, (uint16_t*)Pc, ldpc, vec_p);
            else       hipLaunchKernelGGL((compact_gather_kernel<uint16_t, 2>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc, (const uint16_t*)P, ldp, (uint16_t*)Pc, ldpc, vec_p);
        } else {
            if (vec_q) hipLaunchKernelGGL((compact_gather_kernel<uint32_t, 16>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc, (const uint32_t*)P, ldp, (uint32_t*)Pc, ldpc, vec_p);
            else       hipLaunchKernelGGL((compact_gather_kernel<uint32_t, 4>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc, (const uint32_t*)P, ldp, (uint32_t*)Pc, ldpc, vec_p);
        }
        return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
    }
    if (Qc) {
        const dim3 grid((unsigned)r);
        if (dt == FLOP_BF16) {
            if (vec_q) hipLaunchKernelGGL((compact_rows_kernel<2, 16>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc);
            else       hipLaunchKernelGGL((compact_rows_kernel<2, 2>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc);
        } else {
            if (vec_q) hipLaunchKernelGGL((compact_rows_kernel<4, 16>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc);
            else       hipLaunchKernelGGL((compact_rows_kernel<4, 4>), grid, block, 0, st, Q, ldq, (int)d, (int)r, r_out, idx, zz, absorb_z_into_Q, Qc, ldqc);
        }
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    if (Pc) {
        const dim3 grid((unsigned)dout);
        if (dt == FLOP_BF16)
            hipLaunchKernelGGL(compact_cols_kernel<uint16_t>, grid, block, 0, st, (const uint16_t*)P, ldp, (int)r, r_out, idx, (uint16_t*)Pc, ldpc, vec_p);
        else
            hipLaunchKernelGGL(compact_cols_kernel<uint32_t>, grid, block, 0, st, (const uint32_t*)P, ldp, (int)r, r_out, idx, (uint32_t*)Pc, ldpc, vec_p);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }
    return FLOP_OK;
}

int flop_gate_sample_l0(const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                        float* z, float* dzda, const float* w, float* l0_sum, float* l0_grad,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!valid_hc(hc)) return FLOP_ERR_PARAM;
    if (n_gates < 0 || n_gates > ((int64_t)1 << 40)) return FLOP_ERR_SHAPE;
    if (!l0_sum || (n_gates > 0 && (!log_alpha || !u || !z))) return FLOP_ERR_NULL;
    if (n_gates > 4096) {
        const int rc = flop_gate_sample(log_alpha, u, n_gates, hc, FLOP_GATE_TRAIN, z, dzda, stream);
        if (rc != FLOP_OK) return rc;
        return flop_expected_l0(log_alpha, w, n_gates, hc, l0_sum, l0_grad, workspace, workspace_bytes, stream);
    }
    const float shift = hc.beta * logf(-hc.l / hc.r);
    hipLaunchKernelGGL(gate_l0_kernel, dim3(1), dim3(kGateL0Threads), 0, (hipStream_t)stream, log_alpha, u, w,
                       (int)n_gates, hc.beta, hc.l, hc.r, shift, z, dzda, l0_grad, l0_sum);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_step_boundary(const flop_gate_grad_pending* items, int32_t count,
                       const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                       float* z, float* dzda, const float* w, float* l0_sum, float* l0_grad,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!l0_sum) return FLOP_ERR_NULL;
    const flop_boundary_job j = {nullptr, 0, log_alpha, u, n_gates, hc, z, dzda, w, l0_sum, l0_grad, workspace, workspace_bytes};
    const int rc = boundary_check(items, count, j);
    if (rc != FLOP_OK) return rc;
    return boundary_launch(items, count, j, stream);
}

int flop_bwd_boundary(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* dy, int64_t lddy, const void* x, int64_t ldx,
                      const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                      void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                      float* dlog_alpha, int accumulate,
                      void* workspace, size_t workspace_bytes, const flop_boundary_job* job, void* stream)
{
    if (!job) return FLOP_ERR_NULL;
    int rc = boundary_check(job->items, job->count, *job);
    if (rc != FLOP_OK) return rc;
    if (r > 0 && r <= kMaxDim && z && dlog_alpha) {   // this layer's gate vectors are read by the boundary as well
        const flop_gate_grad_pending own = {(const float*)workspace, z, dzda ? dzda : z, dlog_alpha, nullptr, r, 0, 0};
        rc = boundary_check(&own, 1, *job);
        if (rc != FLOP_OK) return rc;
    }
    return bwd_impl(dt, n, d, r, dout, dy, lddy, x, ldx, Q, ldq, P, ldp, z, dzda, nullptr, g_saved, ldg, dx, lddx,
                    dQ, lddq, dP, lddp, dlog_alpha, accumulate, workspace, workspace_bytes, stream, nullptr, job);
}

int flop_compact(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                 const float* z, const void* Q, int64_t ldq, const void* P, int64_t ldp,
                 int absorb_z_into_Q, int32_t* r_out, int32_t* idx,
                 void* Qc, int64_t ldqc, void* Pc, int64_t ldpc, float* zc,
                 void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    const flop_hc none = {1.0f, -0.1f, 1.1f};
    return compact_impl(dt, d, r, dout, z, Q, ldq, P, ldp, absorb_z_into_Q, r_out, idx, Qc, ldqc, Pc, ldpc, zc,
                        nullptr, nullptr, none, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

int flop_active_prepare(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                        const float* log_alpha, const float* u, flop_hc hc,
                        const void* Q, int64_t ldq, const void* P, int64_t ldp,
                        float* z, float* dzda, int32_t* r_active, int32_t* idx,
                        void* Qc, int64_t ldqc, void* Pc, int64_t ldpc, float* zc, float* dzda_c, void* stream)
{
    if (!valid_hc(hc)) return FLOP_ERR_PARAM;
    if (r > 0 && (!log_alpha || !u)) return FLOP_ERR_NULL;
    return compact_impl(dt, d, r, dout, nullptr, Q, ldq, P, ldp, 0, r_active, idx, Qc, ldqc, Pc, ldpc, zc,
                        log_alpha, u, hc, z, dzda, dzda_c, (hipStream_t)stream);
}

int flop_embed_fwd(flop_dtype dt, int64_t n_tokens, const int64_t* ids, int32_t n_clusters,
                   const flop_embed_cluster* clusters, int64_t d, void* y, int64_t ldy,
                   void* saved, size_t saved_bytes, void* stream)
{
    int64_t dims[kEmbedMaxClusters];
    int rc = validate_embed(dt, n_tokens, n_clusters, clusters, d, dims);
    if (rc != FLOP_OK) return rc;
    if (n_tokens == 0) return FLOP_OK;
    if (!ids || !y || !saved) return FLOP_ERR_NULL;
    if (ldy < d) return FLOP_ERR_STRIDE;
    const EmbedLayout L = embed_layout(dt, n_tokens, d, n_clusters, dims);
    if (saved_bytes < L.saved_total) return FLOP_ERR_WORKSPACE;
    if (((uintptr_t)saved & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    char* sv = (char*)saved;
    int32_t* seg = (int32_t*)(sv + L.seg);
    int32_t* perm = (int32_t*)(sv + L.perm);
    int32_t* rows = (int32_t*)(sv + L.rows);

    EmbedClusterArgs ca;
    memset(&ca, 0, sizeof(ca));
    ca.count = n_clusters;
    for (int c = 0; c < n_clusters; ++c) {
        ca.id_begin[c] = clusters[c].id_begin; ca.id_end[c] = clusters[c].id_end;
        ca.E[c] = clusters[c].E; ca.lde[c] = clusters[c].lde;
        ca.g[c] = sv + L.g[c]; ca.ldg[c] = L.ldg[c];
        ca.z[c] = clusters[c].z; ca.dim[c] = (int)dims[c];
    }
    int n_pow2 = kSortThreads;   // at least one key per thread of the sorting block
    while (n_pow2 < n_tokens) n_pow2 <<= 1;
    // 32-bit keys when the id span and the token positions fit together below the "no cluster" key
    int tok_bits = 0;
    while ((1 << tok_bits) < n_pow2) ++tok_bits;
    const int64_t id_base = clusters[0].id_begin;
    const uint64_t span = (uint64_t)(clusters[n_clusters - 1].id_end - 1 - id_base);
    const bool narrow = (span >> (32 - tok_bits)) == 0 && ((span << tok_bits) | ((1ull << tok_bits) - 1)) < 0xFFFFFFFFull;
    // the 32-bit keys are radix-sorted on their id field, 4 bits a pass: as many passes as it takes for the
    // all-ones "no cluster" key to exceed every id in the bits looked at
    int radix_passes = 1;
    while (radix_passes < 8 && ((1ull << (kRadixBits * radix_passes)) - 1) <= span) ++radix_passes;
    const size_t radix_lds = (size_t)kRadixBuckets * kSortThreads * sizeof(uint16_t);
    auto sort_launch = [&](auto key_tag, auto kpt_tag) -> int {
        using KeyT = decltype(key_tag);
        constexpr int KPT = decltype(kpt_tag)::value;
        static AttrOnce attr;   // one per instantiation of this lambda's call operator
        int sort_dev = 0;
        const size_t lds = (size_t)n_pow2 * sizeof(KeyT) + (sizeof(KeyT) == 4 ? radix_lds : 0);
        if (attr.needed(&sort_dev)) {
            const size_t most = (size_t)kSortThreads * KPT * sizeof(KeyT) + (sizeof(KeyT) == 4 ? radix_lds : 0);
            if (hipFuncSetAttribute((const void*)embed_sort_kernel<KeyT, KPT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)most) != hipSuccess)
                return FLOP_ERR_HIP;
            attr.done(sort_dev);
        }
        hipLaunchKernelGGL((embed_sort_kernel<KeyT, KPT>), dim3(1), dim3(kSortThreads), lds, st, ids, (int)n_tokens, n_pow2, ca,
                           id_base, tok_bits, sizeof(KeyT) == 4 ? radix_passes : 0, perm, rows, seg,
                           (int32_t*)(sv + L.run_start), (int64_t*)(sv + L.uniq_ids), (int32_t*)(sv + L.run_id));
        return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
    };
    auto sort_keys = [&](auto key_tag) -> int {
        switch (n_pow2 / kSortThreads) {
            case 1: return sort_launch(key_tag, std::integral_constant<int, 1>());
            case 2: return sort_launch(key_tag, std::integral_constant<int, 2>());
            case 4: return sort_launch(key_tag, std::integral_constant<int, 4>());
            case 8: return sort_launch(key_tag, std::integral_constant<int, 8>());
            default: return sort_launch(key_tag, std::integral_constant<int, 16>());
        }
    };
    rc = narrow ? sort_keys((unsigned)0) : sort_keys((unsigned long long)0);
    if (rc != FLOP_OK) return rc;
    if (dt == FLOP_BF16)
        hipLaunchKernelGGL(embed_gather_gate_kernel<2>, dim3((unsigned)n_tokens), dim3(128), 0, st, ca, rows, seg);
    else
        hipLaunchKernelGGL(embed_gather_gate_kernel<4>, dim3((unsigned)n_tokens), dim3(128), 0, st, ca, rows, seg);
    if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;

    // y[perm[first_c + i], :] = g_c[i, :] O_c, clusters grouped four to a launch
    for (int c0 = 0; c0 < n_clusters; c0 += kMaxGroup) {
        GemmDesc g[kMaxGroup];
        int cnt = 0;
        for (int c = c0; c < n_clusters && cnt < kMaxGroup; ++c, ++cnt) {
            g[cnt] = {ca.g[c], L.ldg[c], true, clusters[c].O, clusters[c].ldo, false, y, ldy, n_tokens, d, dims[c], nullptr,
                      seg + 2 * c, 1, false, false, false, perm};
        }
        rc = launch_group(dt, g, cnt, st);
        if (rc != FLOP_OK) return rc;
    }
    return FLOP_OK;
}

int flop_embed_bwd(flop_dtype dt, int64_t n_tokens, int32_t n_clusters, const flop_embed_cluster* clusters,
                   int64_t d, const void* dy, int64_t lddy, const void* saved, size_t saved_bytes,
                   int64_t* touched_ids, int32_t* n_touched,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    int64_t dims[kEmbedMaxClusters];
    int rc = validate_embed(dt, n_tokens, n_clusters, clusters, d, dims);
    if (rc != FLOP_OK) return rc;
    for (int c = 0; c < n_clusters; ++c) {
        if (clusters[c].dlog_alpha && !clusters[c].dzda) return FLOP_ERR_NULL;
        if ((clusters[c].dE && clusters[c].ldde < dims[c]) || (clusters[c].dO && clusters[c].lddo < d))
            return FLOP_ERR_STRIDE;
    }
    if (n_tokens > 0 && (!dy || !saved)) return FLOP_ERR_NULL;
    if (n_tokens > 0 && lddy < d) return FLOP_ERR_STRIDE;
    const EmbedLayout L = embed_layout(dt, n_tokens, d, n_clusters, dims);
    if (n_tokens > 0 && saved_bytes < L.saved_total) return FLOP_ERR_WORKSPACE;
    if (!workspace || workspace_bytes < L.ws_total) return FLOP_ERR_WORKSPACE;
    if ((((uintptr_t)workspace | (uintptr_t)saved) & 255u) != 0) return FLOP_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int es = (int)elem_size(dt);
    const char* sv = (const char*)saved;
    char* ws = (char*)workspace;
    const int32_t* seg = (const int32_t*)(sv + L.seg);
    const int32_t* perm = (const int32_t*)(sv + L.perm);
    const int32_t* rows = (const int32_t*)(sv + L.rows);
    void* dy_sorted = ws + L.dy_sorted;

    if (n_tokens > 0) {
        const int vec = aligned16(dy) && (lddy * es) % 16 == 0;
        if (dt == FLOP_BF16)
            hipLaunchKernelGGL(gather_rows_kernel<2>, dim3((unsigned)n_tokens), dim3(kStreamThreads), 0, st, dy, lddy, perm,
                               seg, (int)d, dy_sorted, L.ldds, vec);
        else
            hipLaunchKernelGGL(gather_rows_kernel<4>, dim3((unsigned)n_tokens), dim3(kStreamThreads), 0, st, dy, lddy, perm,
                               seg, (int)d, dy_sorted, L.ldds, vec);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }

    int fused_rows[kEmbedMaxClusters] = {0};   // tile height if the dh_c product left the column sums of dh_c .* g_c
    for (int c0 = 0; c0 < n_clusters; c0 += kMaxGroup) {
        // dh_c = (dy_c O_c^T) .* z_c
        GemmDesc g[kMaxGroup];
        int cnt = 0, first = -1;
        for (int c = c0; c < n_clusters && cnt < kMaxGroup; ++c)
            if (n_tokens > 0) {
                if (first < 0) first = c;
                g[cnt] = {dy_sorted, L.ldds, true, clusters[c].O, clusters[c].ldo, true, ws + L.dh[c], L.ldg[c],
                          n_tokens, dims[c], d, clusters[c].z, seg + 2 * c, 1, true, false, false, nullptr};
                if (clusters[c].dlog_alpha && dt == FLOP_BF16) {
                    g[cnt].dot = sv + L.g[c]; g[cnt].lddot = L.ldg[c]; g[cnt].dot_partial = (float*)(ws + L.partial[c]);
                }
                ++cnt;
            }
        if (cnt) {
            int rows_h = 0;
            rc = launch_group(dt, g, cnt, st, &rows_h);
            if (rc != FLOP_OK) return rc;
            for (int c = first; c < n_clusters && c < first + cnt; ++c)
                if (clusters[c].dlog_alpha && dt == FLOP_BF16) fused_rows[c] = rows_h;
        }
        // dO_c = g_c^T dy_c
        cnt = 0;
        for (int c = c0; c < n_clusters && cnt < kMaxGroup; ++c)
            if (clusters[c].dO)
                g[cnt++] = {sv + L.g[c], L.ldg[c], false, dy_sorted, L.ldds, false, clusters[c].dO, clusters[c].lddo,
                            dims[c], d, n_tokens, nullptr, n_tokens > 0 ? seg + 2 * c : nullptr, 2, false, true, false, nullptr};
        if (cnt) { rc = launch_group(dt, g, cnt, st); if (rc != FLOP_OK) return rc; }
    }

    // gate gradients: dz = (sum_i dh .* g) / z^2 over the cluster's tokens; column sums from the product's
    // epilogue where it gave them, else from the reduction kernel; one finish launch for all clusters
    const int chunks = (int)((n_tokens + kColsumChunkRows - 1) / kColsumChunkRows);
    FinishBatch fb;
    memset(&fb, 0, sizeof(fb));
    int64_t max_r = 0;
    bool any_gate = false;
    for (int c = 0; c < n_clusters; ++c) {
        if (!clusters[c].dlog_alpha) continue;
        float* partial = (float*)(ws + L.partial[c]);
        if (chunks > 0 && !fused_rows[c]) {
            const int cols_per_block = 32 * (16 / es);
            const dim3 grid((unsigned)chunks, (unsigned)((dims[c] + cols_per_block - 1) / cols_per_block));
            if (dt == FLOP_BF16)
                hipLaunchKernelGGL(colsum_dot_kernel<2>, grid, dim3(kStreamThreads), 0, st, (const void*)(ws + L.dh[c]), L.ldg[c],
                                   (const void*)(sv + L.g[c]), L.ldg[c], (int)n_tokens, (int)dims[c], partial, 1, seg + 2 * c, kColsumChunkRows);
            else
                hipLaunchKernelGGL(colsum_dot_kernel<4>, grid, dim3(kStreamThreads), 0, st, (const void*)(ws + L.dh[c]), L.ldg[c],
                                   (const void*)(sv + L.g[c]), L.ldg[c], (int)n_tokens, (int)dims[c], partial, 1, seg + 2 * c, kColsumChunkRows);
            if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
        }
        fb.partial[c] = partial; fb.z[c] = clusters[c].z; fb.dzda[c] = clusters[c].dzda;
        fb.dlog_alpha[c] = clusters[c].dlog_alpha; fb.seg[c] = n_tokens > 0 ? seg + 2 * c : nullptr;
        fb.r[c] = dims[c]; fb.chunks[c] = chunks; fb.chunk_rows[c] = fused_rows[c] ? fused_rows[c] : kColsumChunkRows;
        if (dims[c] > max_r) max_r = dims[c];
        any_gate = true;
    }
    if (any_gate) {
        hipLaunchKernelGGL(dalpha_finish_batch_kernel, dim3((unsigned)((max_r + 31) / 32), (unsigned)n_clusters),
                           dim3(kStreamThreads), 0, st, fb);
        if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
    }

    if (n_tokens > 0) {
        EmbedClusterArgs ca;
        memset(&ca, 0, sizeof(ca));
        ca.count = n_clusters;
        bool any = false;
        for (int c = 0; c < n_clusters; ++c) {
            ca.g[c] = ws + L.dh[c]; ca.ldg[c] = L.ldg[c]; ca.dim[c] = (int)dims[c];
            ca.dE[c] = clusters[c].dE; ca.ldde[c] = clusters[c].ldde;
            any = any || clusters[c].dE;
        }
        if (any) {
            const dim3 grid((unsigned)((n_tokens + kScatterWindow - 1) / kScatterWindow)), block(kScatterThreads);
            const dim3 wgrid(grid.x, (unsigned)((L.ld_scatter + kScatterThreads - 1) / kScatterThreads));
            const int32_t* run_start = (const int32_t*)(sv + L.run_start);
            const int32_t* run_id = (const int32_t*)(sv + L.run_id);
            float* head = (float*)(ws + L.scatter_head);
            float* tail = (float*)(ws + L.scatter_tail);
            if (dt == FLOP_BF16) {
                hipLaunchKernelGGL(embed_scatter_window_kernel<2>, wgrid, block, 0, st, ca, rows, seg, run_start, run_id, head, tail, L.ld_scatter, (int)n_tokens);
                hipLaunchKernelGGL(embed_scatter_join_kernel<2>, grid, block, 0, st, ca, rows, seg, run_start, run_id,
                                   (const float*)head, (const float*)tail, L.ld_scatter, (int)n_tokens);
            } else {
                hipLaunchKernelGGL(embed_scatter_window_kernel<4>, wgrid, block, 0, st, ca, rows, seg, run_start, run_id, head, tail, L.ld_scatter, (int)n_tokens);
                hipLaunchKernelGGL(embed_scatter_join_kernel<4>, grid, block, 0, st, ca, rows, seg, run_start, run_id,
                                   (const float*)head, (const float*)tail, L.ld_scatter, (int)n_tokens);
            }
            if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
        }
        if (touched_ids || n_touched) {
            hipLaunchKernelGGL(embed_touched_kernel, dim3(16), dim3(256), 0, st, (const int64_t*)(sv + L.uniq_ids), seg,
                               touched_ids, n_touched);
            if (hipGetLastError() != hipSuccess) return FLOP_ERR_HIP;
        }
    }
    return FLOP_OK;
}

int flop_bench_phases_begin(void)
{
#ifdef FLOP_PHASE_STAMPS
    if (hipDeviceSynchronize() != hipSuccess) return FLOP_ERR_HIP;
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(flop::g_phase_stamps)) != hipSuccess) return FLOP_ERR_HIP;
    if (hipMemset(p, 0, sizeof(unsigned long long) * kStampSlots * kStampBlocks * kStampPhases) != hipSuccess) return FLOP_ERR_HIP;
    g_stamp_launches.store(0);
    return FLOP_OK;
#else
    return FLOP_ERR_PARAM;
#endif
}

int flop_bench_phases_read(int launch, unsigned long long* stamps, int max_blocks)
{
#ifdef FLOP_PHASE_STAMPS
    if (launch < 0 || launch >= kStampSlots || max_blocks < 0) return FLOP_ERR_SHAPE;
    if (!stamps) return FLOP_ERR_NULL;
    if (hipDeviceSynchronize() != hipSuccess) return FLOP_ERR_HIP;
    const int blocks = max_blocks < kStampBlocks ? max_blocks : kStampBlocks;
    if (hipMemcpyFromSymbol(stamps, HIP_SYMBOL(flop::g_phase_stamps), sizeof(unsigned long long) * blocks * kStampPhases,
                            sizeof(unsigned long long) * (size_t)launch * kStampBlocks * kStampPhases) != hipSuccess)
        return FLOP_ERR_HIP;
    return blocks;
#else
    (void)launch; (void)stamps; (void)max_blocks;
    return FLOP_ERR_PARAM;
#endif
}

}  // extern "C"
