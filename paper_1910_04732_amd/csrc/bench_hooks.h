// What the library's launchers need from the measurement and test aids of flop_bench.h (defined in
// flop_bench.hip): the per-launch trace slots and the forced block shape.
#pragma once

#include <hip/hip_runtime.h>

namespace flop {

struct TraceSlot { hipEvent_t start, stop; int kernel_id; int tiles; double flops; };

// A slot for the launch that is about to be made, or nullptr when tracing is off or the trace is full.
TraceSlot* trace_acquire(int kernel_id, int tiles, double flops);

constexpr int kNumTileShapes = 14;   // block shapes of the bf16 transfer kernel (flop_api.hip: kShapes)

// Block shape every bf16 transfer-kernel launch is to use (flop_bench_force_tile_shape), or -1.
int forced_tile_shape();

}  // namespace flop
