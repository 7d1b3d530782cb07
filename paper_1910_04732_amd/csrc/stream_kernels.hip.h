// Bandwidth-bound kernels of the gated factorized layer: Hard-Concrete gates,
// the expected-L0 sum, the finishing step of the gate gradient, and compaction.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flop {

constexpr int kStreamThreads = 256;

// ---------------------------------------------------------------------------
// Hard-Concrete gate (Section 3): s = sigmoid(t), s-bar = s (r-l) + l,
// z = clamp(s-bar, 0, 1); t = (log u - log(1-u) + alpha)/beta when training,
// t = alpha for the deterministic mask.
// ---------------------------------------------------------------------------
// exp(-t) for the logistic function, with t clamped so that neither e nor 1 + e overflows.
__device__ __forceinline__ float exp_neg_clamped(float t)
{
    return __expf(-fminf(fmaxf(t, -80.0f), 80.0f));
}

// Hardware log2/exp2 based logf/expf (about 1e-6 relative error) keep the kernel
// bound by memory rather than by the transcendental sequences; the stated tolerance
// of the gates is 1e-5 absolute.
__device__ __forceinline__ void gate_one(float a, float u, float inv_beta, float l, float r, int mode,
                                         float& z, float& dzda)
{
    float t, inv_temp;
    if (mode == 0) {
        // log u - log(1 - u) = log(u / (1 - u)); 1 - u is exact for u >= 1/2
        t = (__logf(__fdividef(u, 1.0f - u)) + a) * inv_beta;
        inv_temp = inv_beta;
    } else {
        t = a;
        inv_temp = 1.0f;
    }
    const float e = exp_neg_clamped(t);          // e = exp(-t)
    const float s = __builtin_amdgcn_rcpf(1.0f + e);   // sigmoid(t)
    const float one_minus_s = e * s;             // sigmoid(-t)
    const float sbar = s * (r - l) + l;
    z = fminf(1.0f, fmaxf(0.0f, sbar));
    dzda = (sbar >= 0.0f && sbar <= 1.0f) ? (r - l) * s * one_minus_s * inv_temp : 0.0f;
}

// 16-byte accesses of the streaming kernels.  Stores are marked non-temporal (every byte is written once); loads
// are not: measured on 2^26 gates, past the last-level cache, non-temporal stores gained 3-20 % and cost nothing
// at cache-resident sizes, non-temporal loads gained there too but lost 5-10 % at 2^24 gates.
typedef float f32x4 __attribute__((ext_vector_type(4)));
#ifndef FLOP_NT_LOAD
#define FLOP_NT_LOAD 0
#endif
#ifndef FLOP_NT_STORE
#define FLOP_NT_STORE 1
#endif
__device__ __forceinline__ f32x4 stream_load4(const float* p)
{
#if FLOP_NT_LOAD
    return __builtin_nontemporal_load((const f32x4*)p);
#else
    return *(const f32x4*)p;
#endif
}
__device__ __forceinline__ void stream_store4(float* p, f32x4 v)
{
#if FLOP_NT_STORE
    __builtin_nontemporal_store(v, (f32x4*)p);
#else
    *(f32x4*)p = v;
#endif
}

// VEC = 4: 16-byte accesses (arrays 16-byte aligned); VEC = 1: any alignment.
// A block works on kStreamChunk consecutive gates at a time (UNROLL 16-byte groups per thread, all loads issued
// before the first use), so that each of the four streams is read and written in 16 KB runs.
constexpr int kStreamUnroll = 4;
constexpr int kStreamChunk = kStreamThreads * 4 * kStreamUnroll;

template <int VEC>
__global__ __launch_bounds__(kStreamThreads) void gate_sample_kernel(
    const float* __restrict__ log_alpha, const float* __restrict__ u, int64_t n,
    float beta, float l, float r, int mode, float* __restrict__ z, float* __restrict__ dzda)
{
    constexpr int UNROLL = kStreamUnroll;
    const float inv_beta = 1.0f / beta;
    int64_t done = 0;   // gates covered by whole chunks
    if (VEC == 4) {
        const int64_t chunks = n / kStreamChunk;
        for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
            const int64_t k = c * kStreamChunk + threadIdx.x * 4;
            f32x4 a[UNROLL], uu[UNROLL];
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                a[q] = stream_load4(log_alpha + k + q * (kStreamThreads * 4));
                uu[q] = (mode == 0) ? stream_load4(u + k + q * (kStreamThreads * 4)) : f32x4{0.5f, 0.5f, 0.5f, 0.5f};
            }
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                f32x4 zz, dd;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float ze, de;
                    gate_one(a[q][e], uu[q][e], inv_beta, l, r, mode, ze, de);
                    zz[e] = ze; dd[e] = de;
                }
                stream_store4(z + k + q * (kStreamThreads * 4), zz);
                if (dzda) stream_store4(dzda + k + q * (kStreamThreads * 4), dd);
            }
        }
        done = chunks * kStreamChunk;
    }
    // the rest (less than a chunk when VEC == 4), one group of VEC per thread and pass
    const int64_t stride = (int64_t)gridDim.x * kStreamThreads * VEC;
    for (int64_t k = done + ((int64_t)blockIdx.x * kStreamThreads + threadIdx.x) * VEC; k < n; k += stride) {
        if (VEC == 4 && k + 4 <= n) {
            const f32x4 a = *(const f32x4*)(log_alpha + k);
            f32x4 uu = {0.5f, 0.5f, 0.5f, 0.5f};
            if (mode == 0) uu = *(const f32x4*)(u + k);
            f32x4 zz, dd;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float ze, de;
                gate_one(a[e], uu[e], inv_beta, l, r, mode, ze, de);
                zz[e] = ze; dd[e] = de;
            }
            *(f32x4*)(z + k) = zz;
            if (dzda) *(f32x4*)(dzda + k) = dd;
        } else {
            for (int e = 0; e < VEC && k + e < n; ++e) {
                float zz, dd;
                gate_one(log_alpha[k + e], mode == 0 ? u[k + e] : 0.5f, inv_beta, l, r, mode, zz, dd);
                z[k + e] = zz;
                if (dzda) dzda[k + e] = dd;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Sum of one double per thread over the first `waves` wavefronts of the block (wave shuffles, then
// LDS); every one of them calls, none of the others does.  Result valid in thread 0.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double block_sum(double v, double* lds /* >= waves doubles */, int waves)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double tot = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < waves; ++w) tot += lds[w];
    return tot;
}

// ---------------------------------------------------------------------------
// Expected L0, Eq.(3): sum_k w_k sigmoid(alpha_k - shift), shift = beta log(-l/r).
// Stage 1 writes one double per block; with gridDim.x == 1 it writes the
// final float directly.  Stage 2 adds the per-block values in index order.
// ---------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(kStreamThreads) void expected_l0_kernel(
    const float* __restrict__ log_alpha, const float* __restrict__ w, int64_t n, float shift,
    float* __restrict__ grad, double* __restrict__ block_sums, float* __restrict__ out)
{
    constexpr int UNROLL = kStreamUnroll;
    __shared__ double lds[kStreamThreads / 64];
    double acc = 0.0;
    auto one = [&](float a, float ww, float& g) {
        const float e = exp_neg_clamped(a - shift);
        const float p = __builtin_amdgcn_rcpf(1.0f + e);   // P[z > 0]
        g = ww * p * (e * p);                // w p (1 - p)
        return ww * p;
    };
    int64_t done = 0;
    if (VEC == 4) {   // whole chunks of kStreamChunk consecutive gates per block and pass
        const int64_t chunks = n / kStreamChunk;
        for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
            const int64_t k = c * kStreamChunk + threadIdx.x * 4;
            f32x4 a[UNROLL], ww[UNROLL];
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                a[q] = stream_load4(log_alpha + k + q * (kStreamThreads * 4));
                ww[q] = w ? stream_load4(w + k + q * (kStreamThreads * 4)) : f32x4{1.0f, 1.0f, 1.0f, 1.0f};
            }
#pragma unroll
            for (int q = 0; q < UNROLL; ++q) {
                f32x4 g;
                float part = 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float ge;
                    part += one(a[q][e], ww[q][e], ge);
                    g[e] = ge;
                }
                acc += (double)part;
                if (grad) stream_store4(grad + k + q * (kStreamThreads * 4), g);
            }
        }
        done = chunks * kStreamChunk;
    }
    const int64_t stride = (int64_t)gridDim.x * kStreamThreads * VEC;
    for (int64_t k = done + ((int64_t)blockIdx.x * kStreamThreads + threadIdx.x) * VEC; k < n; k += stride) {
        for (int e = 0; e < VEC && k + e < n; ++e) {
            float g;
            acc += (double)one(log_alpha[k + e], w ? w[k + e] : 1.0f, g);
            if (grad) grad[k + e] = g;
        }
    }
    const double tot = block_sum(acc, lds, kStreamThreads / 64);
    if (threadIdx.x == 0) {
        if (gridDim.x == 1) out[0] = (float)tot;
        else block_sums[blockIdx.x] = tot;
    }
}

__global__ __launch_bounds__(kStreamThreads) void expected_l0_finish_kernel(
    const double* __restrict__ block_sums, int nblocks, float* __restrict__ out)
{
    __shared__ double lds[kStreamThreads / 64];
    double acc = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += kStreamThreads) acc += block_sums[i];
    const double tot = block_sum(acc, lds, kStreamThreads / 64);
    if (threadIdx.x == 0) out[0] = (float)tot;
}

// ---------------------------------------------------------------------------
// Gate gradient, first stage: the column reduction behind
//   dz_k = sum_i dg_ik h_ik = (sum_i dh_ik g_ik) / z_k^2     (dh = dg z, g = h z)
// Block (bx, by) reduces rows [bx*chunk_rows, (bx+1)*chunk_rows) of the 32 column
// groups of 16 bytes numbered by*32..: partial[bx][k] = sum_i A[i,k] * B[i,k].  A wave reads two rows of
// 512 contiguous bytes per step; the eight row lanes of a block are combined
// through LDS in a fixed order, so the result is deterministic.
// ---------------------------------------------------------------------------
constexpr int kColsumChunkRows = 32;   // smallest chunk; sizes the partial buffer

// 16 bytes of A times 16 bytes of B, element-wise, accumulated into acc[16 / ES]
template <int ES>
__device__ __forceinline__ void fma16(const uint4& va, const uint4& vb, float* acc)
{
    const uint32_t wa[4] = {va.x, va.y, va.z, va.w}, wb[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
    for (int e = 0; e < 16 / ES; ++e) {
        float a, b;
        if (ES == 2) {
            a = __builtin_bit_cast(float, (wa[e >> 1] >> (16 * (e & 1))) << 16);
            b = __builtin_bit_cast(float, (wb[e >> 1] >> (16 * (e & 1))) << 16);
        } else {
            a = __builtin_bit_cast(float, wa[e & 3]);
            b = __builtin_bit_cast(float, wb[e & 3]);
        }
        acc[e] += a * b;
    }
}

template <int ES>
__global__ __launch_bounds__(kStreamThreads) void colsum_dot_kernel(
    const void* __restrict__ A, int64_t lda, const void* __restrict__ B, int64_t ldb,
    int n, int r, float* __restrict__ partial, int vec_ok, const int32_t* __restrict__ seg, int chunk_rows)
{
    constexpr int E = 16 / ES;
    if (seg) n = seg[1];   // row count known only on the device (n is then its upper bound)
    __shared__ float red[8][32 * E + 1];
    const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
    const int col = (blockIdx.y * 32 + cg) * E;
    const int row0 = blockIdx.x * chunk_rows;
    const int row1 = min(n, row0 + chunk_rows);
    if (row0 >= n) return;   // uniform for the block
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.0f;
    if (col < r) {
        const char* pa = (const char*)A + ((int64_t)(row0 + rl) * lda + col) * ES;
        const char* pb = (const char*)B + ((int64_t)(row0 + rl) * ldb + col) * ES;
        const int64_t sa = 8 * lda * ES, sb = 8 * ldb * ES;   // the block's eight row lanes step together
        int row = row0 + rl;
        if (vec_ok && col + E <= r) {
            for (; row + 24 < row1; row += 32, pa += 4 * sa, pb += 4 * sb) {   // four rows in flight per lane
                const uint4 a0 = *(const uint4*)pa, a1 = *(const uint4*)(pa + sa), a2 = *(const uint4*)(pa + 2 * sa),
                            a3 = *(const uint4*)(pa + 3 * sa);
                const uint4 b0 = *(const uint4*)pb, b1 = *(const uint4*)(pb + sb), b2 = *(const uint4*)(pb + 2 * sb),
                            b3 = *(const uint4*)(pb + 3 * sb);
                fma16<ES>(a0, b0, acc); fma16<ES>(a1, b1, acc); fma16<ES>(a2, b2, acc); fma16<ES>(a3, b3, acc);
            }
            for (; row < row1; row += 8, pa += sa, pb += sb) fma16<ES>(*(const uint4*)pa, *(const uint4*)pb, acc);
        } else {
            for (; row < row1; row += 8, pa += sa, pb += sb) {
                for (int e = 0; e < E && col + e < r; ++e) {
                    float a, b;
                    if (ES == 2) {
                        a = __builtin_bit_cast(float, (uint32_t)((const uint16_t*)pa)[e] << 16);
                        b = __builtin_bit_cast(float, (uint32_t)((const uint16_t*)pb)[e] << 16);
                    } else {
                        a = ((const float*)pa)[e];
                        b = ((const float*)pb)[e];
                    }
                    acc[e] += a * b;
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < E; ++e) red[rl][cg * E + e] = acc[e];
    __syncthreads();
    const int t = threadIdx.x;
    if (t < 32 * E) {
        const int k = blockIdx.y * 32 * E + t;
        if (k < r) {
            float s = 0.0f;
#pragma unroll
            for (int q = 0; q < 8; ++q) s += red[q][t];
            partial[(int64_t)blockIdx.x * r + k] = s;
        }
    }
}

// ---------------------------------------------------------------------------
// Train-mode gates and the weighted Eq.(3) sum with its gradient in one pass over
// log_alpha, for gate vectors that one block covers (a layer, or a small model): the two
// are the first things every training step needs and read the same array.
// ---------------------------------------------------------------------------
constexpr int kGateL0Threads = 1024;

__global__ __launch_bounds__(kGateL0Threads) void gate_l0_kernel(
    const float* __restrict__ log_alpha, const float* __restrict__ u, const float* __restrict__ w, int n,
    float beta, float l, float r, float shift, float* __restrict__ z, float* __restrict__ dzda,
    float* __restrict__ l0_grad, float* __restrict__ l0_sum)
{
    __shared__ double lds[kGateL0Threads / 64];
    const float inv_beta = 1.0f / beta;
    double acc = 0.0;
    for (int k = threadIdx.x; k < n; k += kGateL0Threads) {
        const float a = log_alpha[k];
        float zz, dd;
        gate_one(a, u[k], inv_beta, l, r, 0, zz, dd);
        z[k] = zz;
        if (dzda) dzda[k] = dd;
        const float ww = w ? w[k] : 1.0f;
        const float e = exp_neg_clamped(a - shift);
        const float p = __builtin_amdgcn_rcpf(1.0f + e);
        if (l0_grad) l0_grad[k] = ww * p * (e * p);
        acc += (double)(ww * p);
    }
    const double tot = block_sum(acc, lds, kGateL0Threads / 64);
    if (threadIdx.x == 0) l0_sum[0] = (float)tot;
}

// ---------------------------------------------------------------------------
// Gate gradient, second stage:
//   dz_k = (sum_c partial[c][k]) / z_k^2
//   dlog_alpha_k = dz_k * dzda_k            (0 where dzda_k == 0 or z_k == 0)
// ---------------------------------------------------------------------------
// A block owns 32 gates; its 8 row lanes add the chunks c = lane, lane+8, ... and
// are combined through LDS in a fixed order.
__device__ __forceinline__ void dalpha_finish_block(
    int block, const float* __restrict__ partial, int chunks, int64_t r, const float* __restrict__ z,
    const float* __restrict__ dzda, float* __restrict__ dlog_alpha, int accumulate,
    const int32_t* __restrict__ seg, int chunk_rows, const int32_t* __restrict__ r_active,
    const int32_t* __restrict__ out_map = nullptr)   // nullable: gate k's result goes to dlog_alpha[out_map[k]], k < r_active
{
    __shared__ double red[8][33];
    if (seg) chunks = (seg[1] + chunk_rows - 1) / chunk_rows;
    const int kl = threadIdx.x & 31, cl = threadIdx.x >> 5;
    const int64_t k = (int64_t)block * 32 + kl;
    // gates beyond the active rank have no partial sums: their gradient is 0
    const int64_t r_used = r_active ? min(r, (int64_t)r_active[0]) : r;
    double s = 0.0;
    if (k < r_used)
        for (int c = cl; c < chunks; c += 8) s += (double)partial[(int64_t)c * r + k];
    red[cl][kl] = s;
    __syncthreads();
    if (cl == 0 && k < r) {
        double tot = 0.0;
#pragma unroll
        for (int q = 0; q < 8; ++q) tot += red[q][kl];
        const float zk = z[k], dk = dzda[k];
        float res = 0.0f;
        if (k < r_used && zk != 0.0f && dk != 0.0f) res = (float)(tot / ((double)zk * (double)zk) * (double)dk);
        if (!out_map) dlog_alpha[k] = accumulate ? dlog_alpha[k] + res : res;
        else if (k < r_used) { const int o = out_map[k]; dlog_alpha[o] = accumulate ? dlog_alpha[o] + res : res; }
    }
}

__global__ __launch_bounds__(kStreamThreads) void dalpha_finish_kernel(
    const float* __restrict__ partial, int chunks, int64_t r, const float* __restrict__ z,
    const float* __restrict__ dzda, float* __restrict__ dlog_alpha, int accumulate,
    const int32_t* __restrict__ seg, int chunk_rows, const int32_t* __restrict__ r_active,
    const int32_t* __restrict__ out_map)
{
    dalpha_finish_block((int)blockIdx.x, partial, chunks, r, z, dzda, dlog_alpha, accumulate, seg, chunk_rows, r_active, out_map);
}

// Up to sixteen gate vectors (the clusters of an adaptive embedding, the layers of a model) in one launch:
// blockIdx.y picks the vector.
constexpr int kFinishBatch = 16;
struct FinishBatch {
    const float* partial[kFinishBatch];
    const float* z[kFinishBatch];
    const float* dzda[kFinishBatch];
    float* dlog_alpha[kFinishBatch];     // NULL: vector absent
    const int32_t* seg[kFinishBatch];
    const int32_t* r_active[kFinishBatch];
    int64_t r[kFinishBatch];
    int chunks[kFinishBatch], chunk_rows[kFinishBatch], accumulate[kFinishBatch];
};

__global__ __launch_bounds__(kStreamThreads) void dalpha_finish_batch_kernel(const FinishBatch b)
{
    const int v = blockIdx.y;
    if (!b.dlog_alpha[v] || (int64_t)blockIdx.x * 32 >= b.r[v]) return;
    dalpha_finish_block((int)blockIdx.x, b.partial[v], b.chunks[v], b.r[v], b.z[v], b.dzda[v], b.dlog_alpha[v],
                        b.accumulate[v], b.seg[v], b.chunk_rows[v], b.r_active[v]);
}

// The boundary between two training steps in one launch: rows 0 .. count-1 of the grid finish the gate
// gradients of the step that ends, block (0, count) samples the gates of the step that begins and adds up
// Eq.(3) (gate vectors of at most 4096 entries).  The new gates go to buffers the finish does not read.
struct GateJob {
    const float* log_alpha; const float* u; const float* w;
    float* z; float* dzda; float* l0_grad; float* l0_sum;
    int n;
    float beta, l, r, shift;
};

// Block (bx, v) of the boundary work; 256 threads.
__device__ __forceinline__ void step_boundary_block(const FinishBatch& b, const int count, const GateJob& gj, int bx, int v)
{
    if (v < count) {
        if (!b.dlog_alpha[v] || (int64_t)bx * 32 >= b.r[v]) return;
        dalpha_finish_block(bx, b.partial[v], b.chunks[v], b.r[v], b.z[v], b.dzda[v], b.dlog_alpha[v],
                            b.accumulate[v], b.seg[v], b.chunk_rows[v], b.r_active[v]);
        return;
    }
    if (bx != 0 || gj.n <= 0) return;
    __shared__ double lds[kStreamThreads / 64];
    const float inv_beta = 1.0f / gj.beta;
    double acc = 0.0;
    for (int k = threadIdx.x; k < gj.n; k += kStreamThreads) {
        const float a = gj.log_alpha[k];
        float zz, dd;
        gate_one(a, gj.u[k], inv_beta, gj.l, gj.r, 0, zz, dd);
        gj.z[k] = zz;
        if (gj.dzda) gj.dzda[k] = dd;
        const float ww = gj.w ? gj.w[k] : 1.0f;
        const float e = exp_neg_clamped(a - gj.shift);
        const float p = __builtin_amdgcn_rcpf(1.0f + e);
        if (gj.l0_grad) gj.l0_grad[k] = ww * p * (e * p);
        acc += (double)(ww * p);
    }
    const double tot = block_sum(acc, lds, kStreamThreads / 64);   // the block may have more wavefronts: they are not here
    if (threadIdx.x == 0) gj.l0_sum[0] = (float)tot;
}

__global__ __launch_bounds__(kStreamThreads) void step_boundary_kernel(const FinishBatch b, const int count, const GateJob gj)
{
    step_boundary_block(b, count, gj, (int)blockIdx.x, (int)blockIdx.y);
}

// The same work as extra blocks of a contraction launch (the last one of a step's backward pass): the
// boundary then costs no launch of its own.  Block id -> (id % bx, id / bx); blocks = bx * (count + 1).
struct BoundaryRider {
    FinishBatch fb;
    GateJob gj;
    int count;
    int bx;        // blocks per gate vector: ceil(largest r / 32)
};

// ---------------------------------------------------------------------------
// Compaction (Sections 4.1 / 4.4): keep k iff z[k] > 0, ascending order.
// One block walks the gates in chunks of blockDim.x; inside a chunk the
// position of a survivor is base + (survivors before it), from wave ballots.
// ---------------------------------------------------------------------------
constexpr int kScanThreads = 1024;

// With log_alpha != NULL the gates are sampled here first (train mode, see gate_one) and written
// to z_out / dzda_out, and dzda of the survivors is gathered to dzc: gate sampling, scan and
// gate gathers of a training step in one launch.  Otherwise z is read.
__global__ __launch_bounds__(kScanThreads) void compact_scan_kernel(
    const float* __restrict__ z, int r, int32_t* __restrict__ r_out, int32_t* __restrict__ idx,
    float* __restrict__ zc,
    const float* __restrict__ log_alpha, const float* __restrict__ u, float beta, float l, float rr,
    float* __restrict__ z_out, float* __restrict__ dzda_out, float* __restrict__ dzc)
{
    __shared__ int wave_count[kScanThreads / 64];
    __shared__ int base_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float inv_beta = 1.0f / beta;
    if (threadIdx.x == 0) base_s = 0;
    __syncthreads();
    for (int start = 0; start < r; start += kScanThreads) {
        const int k = start + threadIdx.x;
        float zk = 0.0f, dk = 0.0f;
        if (k < r) {
            if (log_alpha) {
                gate_one(log_alpha[k], u[k], inv_beta, l, rr, 0, zk, dk);
                if (z_out) z_out[k] = zk;
                if (dzda_out) dzda_out[k] = dk;
            } else {
                zk = z[k];
            }
        }
        const bool keep = zk > 0.0f;
        const unsigned long long mask = __ballot(keep);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_count[wave] = __popcll(mask);
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int wv = 0; wv < kScanThreads / 64; ++wv) {
            const int c = wave_count[wv];
            if (wv < wave) wave_base += c;
            total += c;
        }
        const int base = base_s;
        if (keep) {
            const int pos = base + wave_base + before;
            idx[pos] = k;
            if (zc) zc[pos] = zk;
            if (dzc) dzc[pos] = dk;
        }
        __syncthreads();
        if (threadIdx.x == 0) base_s = base + total;
        __syncthreads();
    }
    const int rp = base_s;
    if (threadIdx.x == 0) r_out[0] = rp;
    if (zc) {
        int pad = (rp + 31) / 32 * 32;
        if (pad > r) pad = r;
        for (int t = rp + threadIdx.x; t < pad; t += kScanThreads) zc[t] = 0.0f;
    }
}

__device__ __forceinline__ uint32_t scale_pack(uint32_t bits, float s, int es)
{
    if (es == 4) return __builtin_bit_cast(uint32_t, __builtin_bit_cast(float, bits) * s);
    const float lo = __builtin_bit_cast(float, bits << 16) * s;
    const float hi = __builtin_bit_cast(float, bits & 0xFFFF0000u) * s;
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)lo) |
           ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)hi) << 16);
}

// Qc[t,:] = Q[idx[t],:] (optionally times z): one block per output row.
// UNIT = bytes per thread access (16 when rows are 16-byte aligned, else ES).
template <int ES, int UNIT>
__device__ __forceinline__ void compact_row_body(
    int t, const void* __restrict__ Q, int64_t ldq, int d, int r, const int32_t* __restrict__ r_out,
    const int32_t* __restrict__ idx, const float* __restrict__ z, int absorb,
    void* __restrict__ Qc, int64_t ldqc)
{
    const int rp = r_out[0];
    int pad = (rp + 31) / 32 * 32;
    if (pad > r) pad = r;
    if (t >= pad) return;
    const int64_t row_bytes = (int64_t)d * ES;
    char* dst = (char*)Qc + (int64_t)t * ldqc * ES;
    if (t >= rp) {
        for (int64_t b = (int64_t)threadIdx.x * UNIT; b < row_bytes; b += (int64_t)kStreamThreads * UNIT) {
            if (UNIT == 16 && b + 16 <= row_bytes) *(uint4*)(dst + b) = uint4{0u, 0u, 0u, 0u};
            else for (int e = 0; e < UNIT && b + e < row_bytes; ++e) dst[b + e] = 0;
        }
        return;
    }
    const int k = idx[t];
    const char* src = (const char*)Q + (int64_t)k * ldq * ES;
    const float s = absorb ? z[k] : 1.0f;
    for (int64_t b = (int64_t)threadIdx.x * UNIT; b < row_bytes; b += (int64_t)kStreamThreads * UNIT) {
        if (UNIT == 16 && b + 16 <= row_bytes) {
            uint4 v = *(const uint4*)(src + b);
            if (absorb) {
                v.x = scale_pack(v.x, s, ES); v.y = scale_pack(v.y, s, ES);
                v.z = scale_pack(v.z, s, ES); v.w = scale_pack(v.w, s, ES);
            }
            *(uint4*)(dst + b) = v;
        } else {
            // element-wise tail / unaligned rows
            for (int64_t e = b; e < b + UNIT && e < row_bytes; e += ES) {
                if (ES == 2) {
                    uint16_t x = *(const uint16_t*)(src + e);
                    if (absorb) x = (uint16_t)scale_pack((uint32_t)x, s, 2);
                    *(uint16_t*)(dst + e) = x;
                } else {
                    uint32_t x = *(const uint32_t*)(src + e);
                    if (absorb) x = scale_pack(x, s, 4);
                    *(uint32_t*)(dst + e) = x;
                }
            }
        }
    }
}

// Pc[m,t] = P[m, idx[t]]: one block per row m.  The row is staged through LDS in pieces of kColChunk source
// columns with 16-byte loads; the survivors of a piece are the index-list range found by binary search (idx is
// ascending), gathered from LDS and written 16 bytes per thread where the output rows allow it (measured: 104 ->
// 93 us on an 8192 x 8192 matrix that keeps 90 % of its columns), else with consecutive lanes on consecutive
// outputs.  The pad columns rp .. pad are zeroed.  16 KB of LDS per block: ten blocks per compute unit keep
// enough loads in flight (32 KB and several rows per block measured slower).
constexpr int kColChunkBytes = 16384;

template <typename U>
__device__ __forceinline__ void compact_col_body(
    int64_t m0, U* __restrict__ lds /* kColChunkBytes of LDS */,
    const U* __restrict__ P, int64_t ldp, int r, const int32_t* __restrict__ r_out,
    const int32_t* __restrict__ idx, U* __restrict__ Pc, int64_t ldpc, int vec_ok)
{
    constexpr int kColChunk = kColChunkBytes / (int)sizeof(U);
    constexpr int E = 16 / (int)sizeof(U);
    const int rp = r_out[0];
    int pad = (rp + 31) / 32 * 32;
    if (pad > r) pad = r;
    const bool out_vec = (((uintptr_t)Pc & 15u) == 0) && ((ldpc * sizeof(U)) % 16 == 0);
    const U* src = P + m0 * ldp;
    U* dst = Pc + m0 * ldpc;
    U* row = lds;
    int t0 = 0;   // first survivor with idx >= chunk start
    for (int c0 = 0; c0 < r && t0 < rp; c0 += kColChunk) {
        const int c1 = min(r, c0 + kColChunk);
        // number of survivors below c1 (same search in every thread; every survivor lies below r, so the last
        // piece - the only one of a row of up to kColChunk columns - needs no search: a dozen dependent loads saved)
        int lo = t0, hi = rp;
        if (c1 >= r) lo = rp;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (idx[mid] < c1) lo = mid + 1; else hi = mid;
        }
        const int t1 = lo;
        if (t1 > t0) {
            if (vec_ok) {
                for (int k = threadIdx.x * E; k < c1 - c0; k += kStreamThreads * E) {
                    if (k + E <= c1 - c0) *(uint4*)(row + k) = *(const uint4*)(src + c0 + k);
                    else for (int e = 0; k + e < c1 - c0; ++e) row[k + e] = src[c0 + k + e];
                }
            } else {
                for (int k = threadIdx.x; k < c1 - c0; k += kStreamThreads) row[k] = src[c0 + k];
            }
            __syncthreads();
            if (out_vec) {
                // whole 16-byte groups of outputs that lie inside [t0, t1); the ragged ends one by one
                const int ta = (t0 + E - 1) / E * E, tb = t1 / E * E;
                if (ta >= tb) {
                    for (int t = t0 + threadIdx.x; t < t1; t += kStreamThreads) dst[t] = row[idx[t] - c0];
                } else {
                    for (int t = t0 + threadIdx.x; t < ta; t += kStreamThreads) dst[t] = row[idx[t] - c0];
                    for (int t = tb + threadIdx.x; t < t1; t += kStreamThreads) dst[t] = row[idx[t] - c0];
                    for (int t = ta + threadIdx.x * E; t < tb; t += kStreamThreads * E) {
                        __attribute__((aligned(16))) U v[E];
#pragma unroll
                        for (int e = 0; e < E; ++e) v[e] = row[idx[t + e] - c0];
                        *(uint4*)(dst + t) = *(const uint4*)v;
                    }
                }
            } else {
                for (int t = t0 + threadIdx.x; t < t1; t += kStreamThreads) dst[t] = row[idx[t] - c0];
            }
            __syncthreads();
        }
        t0 = t1;
    }
    for (int t = rp + threadIdx.x; t < pad; t += kStreamThreads) dst[t] = (U)0;
}

template <int ES, int UNIT>
__global__ __launch_bounds__(kStreamThreads) void compact_rows_kernel(
    const void* __restrict__ Q, int64_t ldq, int d, int r, const int32_t* __restrict__ r_out,
    const int32_t* __restrict__ idx, const float* __restrict__ z, int absorb,
    void* __restrict__ Qc, int64_t ldqc)
{
    compact_row_body<ES, UNIT>((int)blockIdx.x, Q, ldq, d, r, r_out, idx, z, absorb, Qc, ldqc);
}

template <typename U>
__global__ __launch_bounds__(kStreamThreads) void compact_cols_kernel(
    const U* __restrict__ P, int64_t ldp, int r, const int32_t* __restrict__ r_out,
    const int32_t* __restrict__ idx, U* __restrict__ Pc, int64_t ldpc, int vec_ok)
{
    __shared__ __attribute__((aligned(16))) U row[kColChunkBytes / sizeof(U)];
    compact_col_body<U>((int64_t)blockIdx.x, row, P, ldp, r, r_out, idx, Pc, ldpc, vec_ok);
}

// Both gathers in one launch: blocks [0, r) copy rows of Q, blocks [r, r + dout) gather rows of P.
template <typename U, int UNIT>
__global__ __launch_bounds__(kStreamThreads) void compact_gather_kernel(
    const void* __restrict__ Q, int64_t ldq, int d, int r, const int32_t* __restrict__ r_out,
    const int32_t* __restrict__ idx, const float* __restrict__ z, int absorb, void* __restrict__ Qc, int64_t ldqc,
    const U* __restrict__ P, int64_t ldp, U* __restrict__ Pc, int64_t ldpc, int vec_p)
{
    __shared__ __attribute__((aligned(16))) U row[kColChunkBytes / sizeof(U)];
    if ((int)blockIdx.x < r)
        compact_row_body<(int)sizeof(U), UNIT>((int)blockIdx.x, Q, ldq, d, r, r_out, idx, z, absorb, Qc, ldqc);
    else
        compact_col_body<U>((int64_t)blockIdx.x - r, row, P, ldp, r, r_out, idx, Pc, ldpc, vec_p);
}

// ---------------------------------------------------------------------------
// Train-time active ranks (Section 4.3, last paragraph: one mask per batch, so the
// closed components can be left out of the step): helpers around the compacted factors.
// ---------------------------------------------------------------------------
// dst[j] = src[idx[j]] for j < r_active (e.g. dz/dalpha of the surviving gates).
__global__ __launch_bounds__(kStreamThreads) void gather_gates_kernel(
    const float* __restrict__ src, const int32_t* __restrict__ idx, const int32_t* __restrict__ r_active,
    float* __restrict__ dst)
{
    const int rp = r_active[0];
    for (int j = blockIdx.x * kStreamThreads + threadIdx.x; j < rp; j += gridDim.x * kStreamThreads) dst[j] = src[idx[j]];
}

__device__ __forceinline__ int active_slot(const int32_t* __restrict__ idx, int rp, int k);

// Block k (one per component): if k is not in the ascending list idx[0 .. r_active) it is closed, and row k of the
// two gradients a (cols_a columns) and b (cols_b columns), elements of es bytes, and gate[k] are set to zero
// (each output nullable).  The open rows are written by the contractions themselves.
__global__ __launch_bounds__(kStreamThreads) void zero_closed_rows_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ r_active, int r,
    void* __restrict__ a, int64_t lda, int cols_a, void* __restrict__ b, int64_t ldb, int cols_b, int es,
    float* __restrict__ gate)
{
    const int k = blockIdx.x;
    if (k >= r || active_slot(idx, min(r, r_active[0]), k) >= 0) return;
    if (gate && threadIdx.x == 0) gate[k] = 0.0f;
    void* rows[2] = {a, b};
    const int64_t lds_[2] = {lda, ldb};
    const int cols[2] = {cols_a, cols_b};
    for (int q = 0; q < 2; ++q) {
        if (!rows[q]) continue;
        char* dst = (char*)rows[q] + (int64_t)k * lds_[q] * es;
        const int64_t bytes = (int64_t)cols[q] * es;
        if ((((uintptr_t)dst) & 15u) == 0) {
            for (int64_t o = (int64_t)threadIdx.x * 16; o + 16 <= bytes; o += (int64_t)kStreamThreads * 16)
                *(uint4*)(dst + o) = uint4{0u, 0u, 0u, 0u};
            for (int64_t o = bytes / 16 * 16 + threadIdx.x; o < bytes; o += kStreamThreads) dst[o] = 0;
        } else {
            for (int64_t o = threadIdx.x; o < bytes; o += kStreamThreads) dst[o] = 0;
        }
    }
}

// Position of k in the ascending list idx[0..rp), or -1.
__device__ __forceinline__ int active_slot(const int32_t* __restrict__ idx, int rp, int k)
{
    int lo = 0, hi = rp;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (idx[mid] < k) lo = mid + 1; else hi = mid;
    }
    return (lo < rp && idx[lo] == k) ? lo : -1;
}

// Rows of the full-size gradient: dQ[k,:] = dQc[slot(k),:] or 0; dlog_alpha[k] likewise.  One block per k.
template <int ES>
__device__ __forceinline__ void expand_row_body(
    int k, const void* __restrict__ dQc, int64_t lddqc, const float* __restrict__ dalpha_c, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ r_active, int d, void* __restrict__ dQ, int64_t lddq, float* __restrict__ dlog_alpha,
    int vec_ok)
{
    const int j = active_slot(idx, r_active[0], k);
    if (dlog_alpha && threadIdx.x == 0) dlog_alpha[k] = (j >= 0) ? dalpha_c[j] : 0.0f;
    if (!dQ) return;
    char* dst = (char*)dQ + (int64_t)k * lddq * ES;
    const char* src = (const char*)dQc + (int64_t)(j >= 0 ? j : 0) * lddqc * ES;
    const int64_t bytes = (int64_t)d * ES;
    int64_t done = 0;
    if (vec_ok) {
        for (int64_t b = (int64_t)threadIdx.x * 16; b + 16 <= bytes; b += (int64_t)kStreamThreads * 16)
            *(uint4*)(dst + b) = (j >= 0) ? *(const uint4*)(src + b) : uint4{0u, 0u, 0u, 0u};
        done = bytes & ~(int64_t)15;
    }
    for (int64_t b = done + (int64_t)threadIdx.x * ES; b < bytes; b += (int64_t)kStreamThreads * ES) {
        if (ES == 2) *(uint16_t*)(dst + b) = (j >= 0) ? *(const uint16_t*)(src + b) : (uint16_t)0;
        else *(uint32_t*)(dst + b) = (j >= 0) ? *(const uint32_t*)(src + b) : 0u;
    }
}

// Columns of the full-size gradient: dP[m,k] = dPc[m,slot(k)] or 0.  The slot of every k is
// looked up once per block into LDS (r <= kExpandMaxLdsRanks) and then serves kExpandRows rows.
constexpr int kExpandRows = 16;
constexpr int kExpandMaxLdsRanks = 16384;

template <int ES>
__device__ __forceinline__ void expand_col_body(
    int block, int32_t* __restrict__ slot_s,
    const void* __restrict__ dPc, int64_t lddpc, const int32_t* __restrict__ idx, const int32_t* __restrict__ r_active,
    int r, int dout, void* __restrict__ dP, int64_t lddp, int use_lds)
{
    const int rp = r_active[0];
    if (use_lds) {
        for (int k = threadIdx.x; k < r; k += kStreamThreads) slot_s[k] = -1;
        __syncthreads();
        for (int j = threadIdx.x; j < rp; j += kStreamThreads) slot_s[idx[j]] = j;
        __syncthreads();
    }
    const int m0 = block * kExpandRows;
    for (int k = threadIdx.x; k < r; k += kStreamThreads) {
        const int j = use_lds ? slot_s[k] : active_slot(idx, rp, k);
#pragma unroll 4
        for (int m = m0; m < min(m0 + kExpandRows, dout); ++m) {
            if (ES == 2) {
                const uint16_t v = (j >= 0) ? ((const uint16_t*)dPc)[(int64_t)m * lddpc + j] : (uint16_t)0;
                ((uint16_t*)dP)[(int64_t)m * lddp + k] = v;
            } else {
                const uint32_t v = (j >= 0) ? ((const uint32_t*)dPc)[(int64_t)m * lddpc + j] : 0u;
                ((uint32_t*)dP)[(int64_t)m * lddp + k] = v;
            }
        }
    }
}

// The same for 16-byte aligned rows: kExpandVecRows rows of dPc are staged in LDS with 16-byte loads, a thread
// gathers the 16 / ES columns of one output chunk from there and stores 16 bytes (the element-wise form above
// spends one 2-byte load and one 2-byte store per element: 16 us for a 3072 x 768 matrix against 5).
// LDS: r slot entries, then kExpandVecRows rows of round_up(r * ES, 16) bytes.
constexpr int kExpandVecRows = 4;

template <int ES>
__device__ __forceinline__ void expand_col_vec_body(
    int block, int32_t* __restrict__ slot_s,
    const void* __restrict__ dPc, int64_t lddpc, const int32_t* __restrict__ idx, const int32_t* __restrict__ r_active,
    int r, int dout, void* __restrict__ dP, int64_t lddp)
{
    constexpr int E = 16 / ES;
    const int rp = r_active[0];
    const int row_bytes = ((r * ES + 15) / 16) * 16;
    unsigned char* stage = (unsigned char*)(slot_s + ((r + 3) / 4) * 4);
    for (int k = threadIdx.x; k < r; k += kStreamThreads) slot_s[k] = -1;
    __syncthreads();
    for (int j = threadIdx.x; j < rp; j += kStreamThreads) slot_s[idx[j]] = j;
    const int m0 = block * kExpandVecRows;
    const int chunks_in = (rp * ES + 15) / 16;   // a row's last chunk may reach into its padding: lddpc * ES is a multiple of 16
    for (int i = threadIdx.x; i < kExpandVecRows * chunks_in; i += kStreamThreads) {
        const int rr = i / chunks_in, c = i - rr * chunks_in, m = m0 + rr;
        if (m < dout) *(uint4*)(stage + rr * row_bytes + c * 16) = *(const uint4*)((const char*)dPc + (int64_t)m * lddpc * ES + c * 16);
    }
    __syncthreads();
    const int chunks_out = (r + E - 1) / E;
    for (int i = threadIdx.x; i < kExpandVecRows * chunks_out; i += kStreamThreads) {
        const int rr = i / chunks_out, c = i - rr * chunks_out, m = m0 + rr;
        if (m >= dout) continue;
        const int k0 = c * E;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int j = (k0 + e < r) ? slot_s[k0 + e] : -1;
            if (j >= 0) {
                if (ES == 2) w[e >> 1] |= (uint32_t)((const uint16_t*)(stage + rr * row_bytes))[j] << (16 * (e & 1));
                else w[e] = ((const uint32_t*)(stage + rr * row_bytes))[j];
            }
        }
        char* dst = (char*)dP + ((int64_t)m * lddp + k0) * ES;
        if (k0 + E <= r) {
            *(uint4*)dst = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            for (int e = 0; k0 + e < r; ++e) {
                if (ES == 2) ((uint16_t*)dst)[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                else ((uint32_t*)dst)[e] = w[e];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Deterministic inference mask of Section 4.4: every gate scored by its Eq.(3) term
// p_k = sigmoid(alpha_k - shift), the `keep` best kept (z_k = p_k), the others zero.
// p is increasing in alpha, so the ranking is done on alpha (equal alphas: lower
// index first), exactly, as a radix select on the order-preserving integer image of
// the float: four passes of 8 bits find the key of the keep-th largest gate and how
// many gates with that very key are kept; a last pass in index order writes z.
// One block: the gate vectors of a model are a few 10^4 entries.
// keep_dev (nullable): device float, e.g. the expected L0 that flop_expected_l0 wrote;
// then keep = rint(keep_dev[0]).
// ---------------------------------------------------------------------------
constexpr int kSelectThreads = 1024;

__device__ __forceinline__ uint32_t ordered_key(float a)
{
    const uint32_t b = __builtin_bit_cast(uint32_t, a + 0.0f);   // -0 and +0 rank alike
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__global__ __launch_bounds__(kSelectThreads) void topk_mask_kernel(
    const float* __restrict__ log_alpha, int64_t n, int64_t keep_host, const float* __restrict__ keep_dev,
    float shift, float* __restrict__ z, int32_t* __restrict__ kept_out)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned prefix_s;
    __shared__ long long krem_s;
    __shared__ int wave_count[kSelectThreads / 64];
    __shared__ long long base_s;
    const int tid = threadIdx.x;
    long long keep = keep_dev ? (long long)rintf(keep_dev[0]) : (long long)keep_host;
    if (keep < 0) keep = 0;
    if (keep > n) keep = n;
    if (kept_out && tid == 0) kept_out[0] = (int32_t)keep;
    auto p_of = [&](float a) { return __builtin_amdgcn_rcpf(1.0f + exp_neg_clamped(a - shift)); };
    if (keep == 0 || keep == n) {
        for (int64_t i = tid; i < n; i += kSelectThreads) z[i] = keep ? p_of(log_alpha[i]) : 0.0f;
        return;
    }
    if (tid == 0) { prefix_s = 0u; krem_s = keep; base_s = 0; }
    unsigned mask = 0u;
    for (int pass = 0; pass < 4; ++pass) {
        const int sb = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        const unsigned prefix = prefix_s;
        for (int64_t i = tid; i < n; i += kSelectThreads) {
            const uint32_t key = ordered_key(log_alpha[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> sb) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            long long cum = 0, krem = krem_s;
            int digit = 0;
            for (int dg = 255; dg >= 0; --dg) {
                const long long c = hist[dg];
                if (cum + c >= krem) { digit = dg; break; }
                cum += c;
            }
            krem_s = krem - cum;
            prefix_s = prefix | ((unsigned)digit << sb);
        }
        mask |= 0xFFu << sb;
        __syncthreads();
    }
    const unsigned T = prefix_s;
    const long long quota = krem_s;   // gates with key == T that are kept, in index order
    const int lane = tid & 63, wave = tid >> 6;
    for (int64_t start = 0; start < n; start += kSelectThreads) {
        const int64_t i = start + tid;
        uint32_t key = 0u;
        float a = 0.0f;
        if (i < n) { a = log_alpha[i]; key = ordered_key(a); }
        const bool eq = (i < n) && key == T;
        const unsigned long long m = __ballot(eq);
        const int before = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wave_count[wave] = __popcll(m);
        __syncthreads();
        long long wave_base = 0, total = 0;
        for (int wv = 0; wv < kSelectThreads / 64; ++wv) {
            const int c = wave_count[wv];
            if (wv < wave) wave_base += c;
            total += c;
        }
        const long long base = base_s;
        if (i < n) {
            const bool kept = key > T || (eq && base + wave_base + before < quota);
            z[i] = kept ? p_of(a) : 0.0f;
        }
        __syncthreads();
        if (tid == 0) base_s = base + total;
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Augmented-Lagrangian size penalty of Section 4.3 as one streaming pass:
//   viol = scale * s - t,   s = expected model size (device scalar from flop_expected_l0)
//   dlog_alpha_k (+)= (lambda1 + 2 lambda2 viol) * scale * size_grad_k      size_grad_k = w_k p_k (1 - p_k)
//   out = {lambda1 viol + lambda2 viol^2, viol, viol^2}   (penalty, and its gradients for the ascent on lambda)
// 8 bytes read + 4 written per gate (12 read when accumulating).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kStreamThreads) void lagrangian_kernel(
    const float* __restrict__ s_dev, const float* __restrict__ lambda, float scale, float t,
    const float* __restrict__ size_grad, int64_t n, float* __restrict__ dlog_alpha, int accumulate,
    float* __restrict__ out)
{
    const float viol = scale * s_dev[0] - t;
    const float l1 = lambda[0], l2 = lambda[1];
    const float coef = (l1 + 2.0f * l2 * viol) * scale;
    if (out && blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = l1 * viol + l2 * viol * viol;
        out[1] = viol;
        out[2] = viol * viol;
    }
    if (!dlog_alpha) return;
    const int64_t stride = (int64_t)gridDim.x * kStreamThreads;
    for (int64_t k = (int64_t)blockIdx.x * kStreamThreads + threadIdx.x; k < n; k += stride) {
        const float v = coef * size_grad[k];
        dlog_alpha[k] = accumulate ? dlog_alpha[k] + v : v;
    }
}

// ---------------------------------------------------------------------------
// Second stage of a k-split contraction: C[m,n] = round(col_scale[n] * sum_s part[s][m][n]),
// slices added in index order (deterministic).
// ---------------------------------------------------------------------------
template <int ES>
__global__ __launch_bounds__(kStreamThreads) void splitk_reduce_kernel(
    const float* __restrict__ part, int slices, int64_t M, int64_t N, const float* __restrict__ col_scale,
    void* __restrict__ C, int64_t ldc)
{
    const int64_t total = M * N;
    const int64_t stride = (int64_t)gridDim.x * kStreamThreads;
    for (int64_t e = (int64_t)blockIdx.x * kStreamThreads + threadIdx.x; e < total; e += stride) {
        const int64_t row = e / N, col = e - row * N;
        float acc = 0.0f;
        for (int s = 0; s < slices; ++s) acc += part[(int64_t)s * total + e];
        if (col_scale) acc *= col_scale[col];
        if (ES == 2) ((uint16_t*)C)[row * ldc + col] = __builtin_bit_cast(uint16_t, (__bf16)acc);
        else ((float*)C)[row * ldc + col] = acc;
    }
}

// Row and column scatter of the compacted gradients in one launch: blocks [0, r) write rows of dQ
// (and dlog_alpha), the following blocks write kExpandRows rows of dP each.  Either part may be absent.
template <int ES>
__global__ __launch_bounds__(kStreamThreads) void expand_grads_kernel(
    const int32_t* __restrict__ r_active, const int32_t* __restrict__ idx, int r,
    const void* __restrict__ dQc, int64_t lddqc, const float* __restrict__ dalpha_c, int d,
    void* __restrict__ dQ, int64_t lddq, float* __restrict__ dlog_alpha, int vec_q, int row_blocks,
    const void* __restrict__ dPc, int64_t lddpc, int dout, void* __restrict__ dP, int64_t lddp, int use_lds)
{
    extern __shared__ __attribute__((aligned(16))) int32_t slot_s[];
    if ((int)blockIdx.x < row_blocks)
        expand_row_body<ES>((int)blockIdx.x, dQc, lddqc, dalpha_c, idx, r_active, d, dQ, lddq, dlog_alpha, vec_q);
    else if (use_lds == 2)
        expand_col_vec_body<ES>((int)blockIdx.x - row_blocks, slot_s, dPc, lddpc, idx, r_active, r, dout, dP, lddp);
    else
        expand_col_body<ES>((int)blockIdx.x - row_blocks, slot_s, dPc, lddpc, idx, r_active, r, dout, dP, lddp, use_lds);
}

}  // namespace flop
