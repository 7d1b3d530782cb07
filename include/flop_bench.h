/*
 * flop_bench.h - measurement and test aids of the gated factorized layer library.  NOT part of the method and
 * not needed by a user of flop.h: benchmarks use the per-launch trace and the matrix-core probe, tests use the
 * tile-shape override to reach every block shape of the contraction kernel with small inputs.  Unlike the
 * entry points of flop.h these keep process-wide state (a pool of hipEvents, the trace switch, the forced shape),
 * so they are not for use while other threads call the library.
 */
#ifndef FLOP_BENCH_H
#define FLOP_BENCH_H

#include "flop.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-launch timing of the contraction kernel, for benchmarks (not part of the
 * method).  Between flop_trace_begin and flop_trace_end every contraction launch
 * made by flop_fwd / flop_bwd stamps a hipEvent pair at the kernel's begin and
 * end (hipExtLaunchKernelGGL); at most `capacity` launches are recorded.  flop_trace_end waits for the
 * recorded work, fills up to max_records records (host memory) in launch order
 * and writes how many to *count.  kernel_id = 1000 * flop_dtype + mean tile edge,
 * plus 100 for the asynchronous-staging bfloat16 kernel and 10000 per k group beyond the first (e.g. 1228: that
 * kernel with 128x128 tiles, 1196: 128x64, 11180: 64x96 with two k groups, 64: float32 generic kernel with 64x64 tiles); flops = 2 M N K summed over the products
 * of the launch; ms = elapsed time between the two events.  The events are host
 * objects the library keeps for reuse; do not trace while capturing a HIP graph.
 */
typedef struct { int kernel_id; int tiles; double flops; float ms; } flop_trace_record;
int flop_trace_begin(int capacity);
int flop_trace_end(flop_trace_record* out, int max_records, int* count);

/*
 * Matrix-core rate probe, for benchmarks (not part of the method): `blocks` workgroups of four
 * wavefronts each issue `iters` rounds of four independent 32x32 matrix instructions of the given type
 * (bfloat16: 32x32x16, float32: 32x32x2) on register operands and nothing else.  The caller times the
 * launch; *flops (host, nullable) receives the flop count of the launch.  sink: device, at least 64
 * floats, overwritten.  FLOP_ERR_SHAPE for iters outside 1..2^24 or blocks outside 1..65536.
 */
int flop_mfma_probe(flop_dtype dt, int64_t iters, int32_t blocks, float* sink, double* flops, void* stream);

/*
 * Forces the block shape of every following launch of the bfloat16 asynchronous-transfer contraction kernel
 * (rows at least 16-byte aligned; other launches are unaffected): shape = 0 .. flop_bench_tile_shapes() - 1, or
 * -1 to give the choice back to the library.  flop_bench_tile_shape_name(shape) describes a shape
 * ("64x96 g2": 64 x 96 tile, two k groups).  Results do not depend on the shape beyond float32 summation order.
 */
int flop_bench_force_tile_shape(int shape);

/*
 * Per-block phase times of the bfloat16 transfer kernel, in the measurement build of the library only
 * (paper_1910_04732_amd/libflop_hip_phases.so: the same sources compiled with -DFLOP_PHASE_STAMPS, in which the
 * first thread of every block records the 100 MHz wall clock at block entry, before its main loop, after it, after
 * its output tile is staged in LDS, and after its stores have completed).  flop_bench_phases_begin() clears the
 * record and restarts the launch count: the following launches of that kernel take the slots 0, 1, ... 15 in
 * order (later launches and blocks beyond 4096 per launch are not recorded).  flop_bench_phases_read(launch,
 * stamps, max_blocks) synchronises the device and copies 5 stamps per block of that launch to host memory (all
 * zero for a block that recorded nothing: padding blocks, riders, k-split launches); returns the number of blocks
 * copied.  In the product library (no stamps compiled in) both return FLOP_ERR_PARAM.
 */
int flop_bench_phases_begin(void);
int flop_bench_phases_read(int launch, unsigned long long* stamps, int max_blocks);
int flop_bench_tile_shapes(void);
const char* flop_bench_tile_shape_name(int shape);

#ifdef __cplusplus
}
#endif
#endif /* FLOP_BENCH_H */
