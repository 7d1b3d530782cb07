// Host stand-in for <hip/hip_runtime.h>, used only by the address model (tests/host_model/address_model.cpp).
//
// The library's single translation unit is compiled for the host CPU with this header in place of HIP's:
// kernels become plain functions, a launch becomes a loop over blocks and threads that runs every thread
// to completion, one after the other, and "device" pointers are ordinary heap pointers.  Under
// AddressSanitizer every global-memory access a thread makes - direct loads and stores, and the
// global -> LDS buffer transfers emulated below - is then checked against the exact extent of the
// allocation it falls in.
//
// What the model keeps: all index and address arithmetic of host and device code, as compiled from the
// product sources.  What it drops: values.  Threads do not run in lockstep, so barriers are no-ops, wave
// shuffles return the caller's own value, matrix instructions return their accumulator, LDS holds
// whatever the last writer left, and static __shared__ arrays are per-thread locals.  Only kernels whose
// addresses do not depend on such values are meaningful here (the contraction kernels, the store-bound kernel for small ranks, the gate, Eq.(3) and
// gate-gradient kernels and the step-boundary blocks); the driver launches nothing else.
#pragma once

#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

// ---- qualifiers ----------------------------------------------------------------------------------------
#define __device__
#define __global__
#define __host__
#define __forceinline__ inline __attribute__((always_inline))
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) (&(x))
#define __shared__   /* static LDS: a per-thread local (values are not modelled); extern LDS: see flop::smem */

// inline assembly (LDS fragment reads, wait counters) carries no global address: dropped.  Every statement
// in the sources is spelled `asm volatile(...)`; `volatile` as a plain qualifier is left alone.
#define asm
#define volatile(...) ((void)0)

// ---- vector types ----------------------------------------------------------------------------------------
struct float2 { float x, y; };
struct float4 { float x, y, z, w; };
struct uint2 { uint32_t x, y; };
struct uint4 { uint32_t x, y, z, w; };
inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return uint4{x, y, z, w}; }

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
inline dim3 threadIdx, blockIdx, blockDim, gridDim;

using std::max;
using std::min;

// ---- runtime API -----------------------------------------------------------------------------------------
typedef void* hipStream_t;
typedef void* hipEvent_t;
enum hipError_t { hipSuccess = 0, hipErrorUnknown = 999 };
enum hipFuncAttribute { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, hipFuncAttribute, int) { return hipSuccess; }
inline hipError_t hipGetSymbolAddress(void** p, const void* symbol) { *p = (void*)symbol; return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t* e) { *e = nullptr; return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }

namespace flop_model {

// Dynamic LDS of the running block.  160 KB, the compute unit's; the launch's own size is enforced by the
// checks in lds_range().
constexpr size_t kLdsBytes = 160 * 1024;
struct Launch {
    size_t lds_bytes = 0;        // dynamic LDS the launch asked for
    unsigned long launches = 0, blocks = 0, transfers = 0, transfers_zero_filled = 0;
};
inline Launch g_launch;

[[noreturn]] inline void fail(const char* what, long a = 0, long b = 0)
{
    fprintf(stderr, "address model: %s (%ld, %ld) in block %u thread %u\n", what, a, b, blockIdx.x, threadIdx.x);
    abort();
}

// A buffer descriptor as the transfer instructions use it: base address and range in bytes.
struct Rsrc { const char* base; uint32_t range; };
inline Rsrc make_rsrc(const void* p, int num_records)
{
    if (num_records < 0) fail("descriptor range negative", num_records);
    return Rsrc{(const char*)p, (uint32_t)num_records};
}

}  // namespace flop_model

namespace flop {
// the extern __shared__ arrays of the kernels
alignas(1024) inline unsigned char smem[flop_model::kLdsBytes];
alignas(16) inline unsigned char smem_raw[flop_model::kLdsBytes];
alignas(16) inline int32_t slot_s[flop_model::kLdsBytes / 4];
}  // namespace flop

namespace flop_model {

// raw_buffer_load ... lds: every lane moves `size` bytes from base + voffset + soffset + inst_offset to
// lds_base + inst_offset' + lane * size.  An access whose last byte lies beyond the descriptor's range
// moves zeros instead (that is the zero-fill the kernels rely on).  The 32-bit offset sum is taken
// without wrap-around here; a sum of 2^32 or more is reported, since the kernels never intend one.
template <typename LdsPtr>
inline void buffer_load_lds(Rsrc r, LdsPtr lds, int size, uint32_t voffset, uint32_t soffset, int inst_offset, int)
{
    unsigned char* dst = (unsigned char*)lds + (threadIdx.x & 63u) * (unsigned)size;
    if (dst < flop::smem || dst + size > flop::smem + g_launch.lds_bytes)
        fail("transfer lands outside the launch's dynamic LDS", (long)(dst - flop::smem), size);
    const uint64_t off = (uint64_t)voffset + soffset + (uint64_t)inst_offset;
    if (off >= (1ull << 32)) fail("transfer offset wraps 32 bits", (long)voffset, (long)soffset);
    ++g_launch.transfers;
    if (off + (uint64_t)size > r.range) {
        memset(dst, 0, (size_t)size);
        ++g_launch.transfers_zero_filled;
    } else {
        memcpy(dst, r.base + off, (size_t)size);   // checked by the sanitizer against the operand's allocation
    }
}

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, Args&&... args)
{
    if (lds > kLdsBytes) fail("dynamic LDS beyond 160 KB", (long)lds);
    g_launch.lds_bytes = lds;
    ++g_launch.launches;
    gridDim = grid;
    blockDim = block;
    for (unsigned bz = 0; bz < grid.z; ++bz)
        for (unsigned by = 0; by < grid.y; ++by)
            for (unsigned bx = 0; bx < grid.x; ++bx) {
                ++g_launch.blocks;
                blockIdx = dim3(bx, by, bz);
                for (unsigned tz = 0; tz < block.z; ++tz)
                    for (unsigned ty = 0; ty < block.y; ++ty)
                        for (unsigned tx = 0; tx < block.x; ++tx) {
                            threadIdx = dim3(tx, ty, tz);
                            kernel(KArgs(args)...);
                        }
            }
}

}  // namespace flop_model

template <typename... KArgs, typename... Args>
inline void hipLaunchKernelGGL(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t, Args&&... args)
{
    flop_model::launch(kernel, grid, block, lds, std::forward<Args>(args)...);
}
template <typename... KArgs, typename... Args>
inline void hipExtLaunchKernelGGL(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t, hipEvent_t,
                                  hipEvent_t, int, Args&&... args)
{
    flop_model::launch(kernel, grid, block, lds, std::forward<Args>(args)...);
}

// ---- device intrinsics: values are not modelled ----------------------------------------------------------
inline void __syncthreads() {}
template <typename T> inline T __shfl_xor(T v, int) { return v; }
template <typename T> inline T __shfl_down(T v, int) { return v; }
inline unsigned long long __ballot(bool p) { return p ? (1ull << (threadIdx.x & 63u)) : 0ull; }
inline int __popcll(unsigned long long v) { return __builtin_popcountll(v); }
template <typename T> inline T atomicAdd(T* p, T v) { T old = *p; *p = old + v; return old; }
inline float __expf(float x) { return expf(x); }
inline float __logf(float x) { return logf(x); }
inline float __fdividef(float a, float b) { return a / b; }

#define __amdgpu_buffer_rsrc_t flop_model::Rsrc
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, num, flags) flop_model::make_rsrc((p), (num))
#define __builtin_amdgcn_raw_ptr_buffer_load_lds(r, lds, size, voff, soff, ioff, aux) \
    flop_model::buffer_load_lds((r), (lds), (size), (voff), (soff), (ioff), (aux))
#define __builtin_amdgcn_s_waitcnt(x) ((void)0)
#define __builtin_amdgcn_s_barrier() ((void)0)
#define __builtin_amdgcn_wave_barrier() ((void)0)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __builtin_amdgcn_update_dpp(old, v, ctrl, rm, bm, bc) (v)
#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) ((void)(a), (void)(b), (c))
#define __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, x, y, z) ((void)(a), (void)(b), (c))

// LDS pointers are ordinary pointers here
#define FLOP_LDS_PTR(p) ((void*)(p))
