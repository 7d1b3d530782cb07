// Measurement and test aids (include/flop_bench.h): per-launch trace of the contraction kernels, the
// matrix-core rate probe, the forced block shape.  A translation unit of its own: nothing here is needed to
// compute anything, and all process-wide state of the library lives here.
#include "../../include/flop_bench.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "bench_hooks.h"

namespace flop {

namespace {
struct TraceState {
    std::mutex mu;
    std::atomic<bool> on{false};
    std::vector<TraceSlot> slots;   // events are created once and reused
    size_t used = 0, capacity = 0;
} g_trace;
std::atomic<int> g_forced_shape{-1};
}  // namespace

TraceSlot* trace_acquire(int kernel_id, int tiles, double flops)
{
    if (!g_trace.on.load(std::memory_order_relaxed)) return nullptr;
    std::lock_guard<std::mutex> lk(g_trace.mu);
    if (!g_trace.on || g_trace.used >= g_trace.capacity) return nullptr;
    TraceSlot* s = &g_trace.slots[g_trace.used++];
    s->kernel_id = kernel_id; s->tiles = tiles; s->flops = flops;
    return s;
}

int forced_tile_shape() { return g_forced_shape.load(std::memory_order_relaxed); }

// ---------------------------------------------------------------------------
// Matrix-core rate probe: every wave issues
// `iters` rounds of four independent 32x32 MFMAs on register operands, nothing else; the
// accumulators are folded into `sink` so the loop cannot be dropped.  The contraction kernels' rate is
// quoted against what this reaches as well as against the datasheet figure.
// ---------------------------------------------------------------------------
constexpr int kProbeWavesPerBlock = 4;
constexpr int kProbeChains = 4;

template <bool BF16>
__global__ __launch_bounds__(64 * kProbeWavesPerBlock) void mfma_probe_kernel(int iters, float* __restrict__ sink)
{
    typedef float acc16 __attribute__((ext_vector_type(16)));
    typedef __bf16 op8 __attribute__((ext_vector_type(8)));
    acc16 acc[kProbeChains];
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.0f;
    // operands small enough that no accumulator leaves the normal range
    const float seed = 1.0f / (float)(1 + (threadIdx.x & 7));
    op8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed * 0.001f); b[e] = (__bf16)(0.5f - seed); }
    const float af = seed * 0.001f, bf = 0.5f - seed;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kProbeChains; ++c) {
            if constexpr (BF16) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
            else                acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc[c], 0, 0, 0);
        }
    }
    float tot = 0.0f;
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) tot += acc[c][e];
    if (blockIdx.x == 0 && threadIdx.x < 64) sink[threadIdx.x] = tot;
}

}  // namespace flop

using namespace flop;

extern "C" {

int flop_mfma_probe(flop_dtype dt, int64_t iters, int32_t blocks, float* sink, double* flops, void* stream)
{
    if (dt != FLOP_F32 && dt != FLOP_BF16) return FLOP_ERR_DTYPE;
    if (iters <= 0 || iters > (1 << 24) || blocks <= 0 || blocks > (1 << 16)) return FLOP_ERR_SHAPE;
    if (!sink) return FLOP_ERR_NULL;
    const double per_mfma = dt == FLOP_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    if (flops) *flops = per_mfma * kProbeChains * (double)iters * kProbeWavesPerBlock * blocks;
    if (dt == FLOP_BF16)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)blocks), dim3(64 * kProbeWavesPerBlock), 0, (hipStream_t)stream,
                           (int)iters, sink);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)blocks), dim3(64 * kProbeWavesPerBlock), 0, (hipStream_t)stream,
                           (int)iters, sink);
    return hipGetLastError() == hipSuccess ? FLOP_OK : FLOP_ERR_HIP;
}

int flop_trace_begin(int capacity)
{
    if (capacity <= 0 || capacity > (1 << 20)) return FLOP_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_trace.mu);
    while (g_trace.slots.size() < (size_t)capacity) {
        TraceSlot s{};
        if (hipEventCreate(&s.start) != hipSuccess || hipEventCreate(&s.stop) != hipSuccess) return FLOP_ERR_HIP;
        g_trace.slots.push_back(s);
    }
    g_trace.capacity = (size_t)capacity;
    g_trace.used = 0;
    g_trace.on = true;
    return FLOP_OK;
}

int flop_trace_end(flop_trace_record* out, int max_records, int* count)
{
    if (!count || (max_records > 0 && !out)) return FLOP_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_trace.mu);
    g_trace.on = false;
    int n = 0;
    for (size_t i = 0; i < g_trace.used && n < max_records; ++i) {
        TraceSlot& s = g_trace.slots[i];
        if (hipEventSynchronize(s.stop) != hipSuccess) return FLOP_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, s.start, s.stop) != hipSuccess) return FLOP_ERR_HIP;
        out[n].kernel_id = s.kernel_id; out[n].tiles = s.tiles; out[n].flops = s.flops; out[n].ms = ms;
        ++n;
    }
    *count = n;
    g_trace.used = 0;
    return FLOP_OK;
}

static const char* const kShapeNames[] = {"128x128", "128x64", "64x64", "64x64 g2", "64x96 g2", "128x64 g2", "128x128 g2",
                                          "256x128", "64x64 g4", "64x96", "64x64 g2 n2", "64x96 g2 n2", "128x64 g2 n2", "64x64 n2"};

static_assert(sizeof(kShapeNames) / sizeof(kShapeNames[0]) == kNumTileShapes, "one name per shape");

int flop_bench_tile_shapes(void) { return kNumTileShapes; }

const char* flop_bench_tile_shape_name(int shape)
{
    return (shape >= 0 && shape < flop_bench_tile_shapes()) ? kShapeNames[shape] : "automatic";
}

int flop_bench_force_tile_shape(int shape)
{
    if (shape < -1 || shape >= flop_bench_tile_shapes()) return FLOP_ERR_SHAPE;
    g_forced_shape.store(shape);
    return FLOP_OK;
}

}  // extern "C"
