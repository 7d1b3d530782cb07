// Kernels of the gated adaptive embedding (Section 4.2): cluster c owns the
// vocabulary ids [id_begin, id_end), a table E_c[n_c, d_c], a projection
// O_c[d_c, d] and gates z_c; the embedding of id t is (E_c[t - id_begin,:] .* z_c) O_c.
//
// Token ids are sorted once per batch (one block, bitonic network in LDS, keys
// id << 32 | token so that equal ids keep token order).  Sorting makes every
// cluster's tokens contiguous, which turns the per-cluster products into dense
// contractions over a run-time segment, and makes repeated words adjacent, so
// that the embedding gradient is a segmented sum in a fixed order (deterministic,
// no floating-point atomics).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stream_kernels.hip.h"

namespace flop {
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kEmbedMaxClusters = 8;
constexpr int kEmbedMaxTokens = 16384;   // one block sorts the batch in LDS (8 bytes per key)
constexpr int kSortThreads = 1024;

struct EmbedClusterArgs {
    int64_t id_begin[kEmbedMaxClusters], id_end[kEmbedMaxClusters];
    const void* E[kEmbedMaxClusters];
    int64_t lde[kEmbedMaxClusters];
    void* g[kEmbedMaxClusters];        // fwd: gathered gated rows; scatter: dh_c
    int64_t ldg[kEmbedMaxClusters];
    const float* z[kEmbedMaxClusters];
    void* dE[kEmbedMaxClusters];
    int64_t ldde[kEmbedMaxClusters];
    int dim[kEmbedMaxClusters];
    int count;
};

// seg[2c] = first sorted position of cluster c, seg[2c+1] = its token count;
// seg[2*kEmbedMaxClusters] = number of distinct ids, seg[2*kEmbedMaxClusters+1] = valid tokens.
constexpr int kSegUnique = 2 * kEmbedMaxClusters;
constexpr int kSegValid = 2 * kEmbedMaxClusters + 1;
constexpr int kSegInts = 2 * kEmbedMaxClusters + 2;

__device__ __forceinline__ int cluster_of(const EmbedClusterArgs& cl, int64_t id)
{
    int c = -1;
#pragma unroll
    for (int q = 0; q < kEmbedMaxClusters; ++q)
        if (q < cl.count && id >= cl.id_begin[q] && id < cl.id_end[q]) c = q;
    return c;
}

// Sorted position -> cluster, from the segment table.
__device__ __forceinline__ int cluster_at(const int32_t* seg, int count, int pos)
{
    int c = -1;
    for (int q = 0; q < count; ++q)
        if (pos >= seg[2 * q] && pos < seg[2 * q] + seg[2 * q + 1]) c = q;
    return c;
}

// Sorts key[0 .. n_pow2) in LDS ascending; n_pow2 = KPT * kSortThreads.  All threads call.
__device__ __forceinline__ unsigned long long shfl_xor_key(unsigned long long v, int lane_xor)
{
    const unsigned lo = __shfl_xor((unsigned)(v & 0xFFFFFFFFull), lane_xor);
    const unsigned hi = __shfl_xor((unsigned)(v >> 32), lane_xor);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned shfl_xor_key(unsigned v, int lane_xor) { return __shfl_xor(v, lane_xor); }

// Lane exchange inside a quad on the vector ALU (no LDS crossbar): quad_perm [1,0,3,2] and [2,3,0,1].
__device__ __forceinline__ unsigned quad_xor1(unsigned v) { return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true); }
__device__ __forceinline__ unsigned quad_xor2(unsigned v) { return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true); }
__device__ __forceinline__ unsigned long long quad_xor1(unsigned long long v)
{
    return ((unsigned long long)quad_xor1((unsigned)(v >> 32)) << 32) | quad_xor1((unsigned)(v & 0xFFFFFFFFull));
}
__device__ __forceinline__ unsigned long long quad_xor2(unsigned long long v)
{
    return ((unsigned long long)quad_xor2((unsigned)(v >> 32)) << 32) | quad_xor2((unsigned)(v & 0xFFFFFFFFull));
}

template <int KPT, typename KeyT>
__device__ __forceinline__ void bitonic_sort_block(KeyT* key, int n_pow2)
{
    const int tid = threadIdx.x;
    KeyT k[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) k[j] = key[tid * KPT + j];
    __syncthreads();
    const int e0 = tid * KPT;   // first key of this thread; bits of e0 + j at or above KPT do not depend on j
    for (int size = 2; size <= n_pow2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride >= KPT) {
                // partner in another thread; the same decision for all keys of this thread
                const bool take_min = ((e0 & stride) == 0) == ((e0 & size) == 0);
                if (stride >= KPT * 64) {   // another wave: through LDS
#pragma unroll
                    for (int j = 0; j < KPT; ++j) key[e0 + j] = k[j];
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < KPT; ++j) {
                        const KeyT p = key[(e0 + j) ^ stride];
                        const KeyT lo = p < k[j] ? p : k[j], hi = p < k[j] ? k[j] : p;
                        k[j] = take_min ? lo : hi;
                    }
                    __syncthreads();
                } else {                    // same wave: lane shuffle
                    const int lane_xor = stride / KPT;
                    KeyT p[KPT];
                    if (lane_xor == 1) {
#pragma unroll
                        for (int j = 0; j < KPT; ++j) p[j] = quad_xor1(k[j]);
                    } else if (lane_xor == 2) {
#pragma unroll
                        for (int j = 0; j < KPT; ++j) p[j] = quad_xor2(k[j]);
                    } else {
#pragma unroll
                        for (int j = 0; j < KPT; ++j) p[j] = shfl_xor_key(k[j], lane_xor);
                    }
#pragma unroll
                    for (int j = 0; j < KPT; ++j) {
                        const KeyT lo = p[j] < k[j] ? p[j] : k[j], hi = p[j] < k[j] ? k[j] : p[j];
                        k[j] = take_min ? lo : hi;
                    }
                }
            } else {
                // the remaining strides of this size lie inside the thread: compile-time register pairs
#pragma unroll
                for (int st = KPT / 2; st > 0; st >>= 1) {
                    if (st > stride) continue;
#pragma unroll
                    for (int j = 0; j < KPT; ++j) {
                        if ((j & st) == 0) {
                            const bool up = ((e0 + j) & size) == 0;
                            const KeyT a = k[j], b = k[j ^ st];
                            const KeyT lo = a < b ? a : b, hi = a < b ? b : a;
                            k[j] = up ? lo : hi;
                            k[j ^ st] = up ? hi : lo;
                        }
                    }
                }
                break;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < KPT; ++j) key[tid * KPT + j] = k[j];
    __syncthreads();
}

// Inclusive scan over the 64 lanes of a wave on the vector ALU (DPP row shifts inside each row of 16 lanes, then
// row broadcasts of the row totals); no LDS crossbar round trips.  Lane layout checked on the device.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1 (shifted-in lanes read 0)
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Stable least-significant-digit radix sort of key[0 .. n_pow2) on bits [bit0, bit0 + 4 * passes), for the
// 32-bit keys: the token position in the low bits is the initial order, so sorting on the id field alone with a
// stable sort gives the order of the full key, in passes of 4 bits instead of log^2(n) compare-exchange stages.
// Thread t owns positions t*KPT .. t*KPT+KPT-1 and column t of a 16 x kSortThreads table of 16-bit counters
// (`cnt`, 32 KB of LDS): it counts its keys per digit in registers, the table is scanned in (digit, thread) order — which is
// (digit, position) order — and a key's rank is its column's scanned entry plus its rank among the thread's own
// keys of that digit.  Counter (d, t) lives in bank (t / 2) % 64 whatever d is: no bank conflicts on the counting.
constexpr int kRadixBits = 4, kRadixBuckets = 1 << kRadixBits;

template <int KPT>
__device__ __forceinline__ void radix_sort_block(unsigned* key, uint16_t* cnt, int* wave_total, int bit0, int passes)
{
    static_assert(KPT >= 1 && KPT <= 16 && kSortThreads * 16 < 65536, "16-bit counters");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned k[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) k[j] = key[tid * KPT + j];
    for (int pass = 0; pass < passes; ++pass) {
        const int shift = bit0 + kRadixBits * pass;
        // per-digit counts of this thread's keys, 8 bits each in two 64-bit registers (at most 16 keys)
        unsigned long long c_lo = 0, c_hi = 0;
        uint16_t own[KPT];   // rank among this thread's keys of the same digit
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const unsigned d = (k[j] >> shift) & (kRadixBuckets - 1);
            const unsigned s8 = (d & 7u) * 8u;
            const bool high = d >= 8u;
            own[j] = (uint16_t)(((high ? c_hi : c_lo) >> s8) & 0xFFull);
            const unsigned long long one = 1ull << s8;
            c_lo += high ? 0ull : one;
            c_hi += high ? one : 0ull;
        }
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            cnt[d * kSortThreads + tid] = (uint16_t)((c_lo >> (8 * d)) & 0xFFull);
            cnt[(d + 8) * kSortThreads + tid] = (uint16_t)((c_hi >> (8 * d)) & 0xFFull);
        }
        __syncthreads();
        // exclusive scan of the flattened table; this thread scans entries 16*tid .. 16*tid+15
        u32x4 w0 = ((const u32x4*)cnt)[tid * 2], w1 = ((const u32x4*)cnt)[tid * 2 + 1];
        unsigned v[16];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = w0[e] & 0xFFFFu; v[2 * e + 1] = w0[e] >> 16;
            v[8 + 2 * e] = w1[e] & 0xFFFFu; v[8 + 2 * e + 1] = w1[e] >> 16;
        }
        unsigned sum = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) { const unsigned t = v[e]; v[e] = sum; sum += t; }
        const unsigned incl = (unsigned)wave_inclusive_scan((int)sum);
        if (lane == 63) wave_total[wave] = (int)incl;
        __syncthreads();
        unsigned before = incl - sum;
#pragma unroll
        for (int wv = 0; wv < kSortThreads / 64; ++wv) {   // all totals are read (fixed addresses), earlier waves count
            const unsigned c = (unsigned)wave_total[wv];
            before += wv < wave ? c : 0u;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w0[e] = ((v[2 * e] + before) & 0xFFFFu) | ((v[2 * e + 1] + before) << 16);
            w1[e] = ((v[8 + 2 * e] + before) & 0xFFFFu) | ((v[8 + 2 * e + 1] + before) << 16);
        }
        ((u32x4*)cnt)[tid * 2] = w0;
        ((u32x4*)cnt)[tid * 2 + 1] = w1;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const int d = (int)((k[j] >> shift) & (kRadixBuckets - 1));
            key[(int)cnt[d * kSortThreads + tid] + (int)own[j]] = k[j];
        }
        __syncthreads();
        if (pass + 1 < passes) {
#pragma unroll
            for (int j = 0; j < KPT; ++j) k[j] = key[tid * KPT + j];
        }
    }
}

// Shared state of the sorting block.
struct SortShared {
    int first[kEmbedMaxClusters], last[kEmbedMaxClusters];
    int wave_count[kSortThreads / 64];
    int valid;
};

// Body of the sorting block for KPT keys per thread: thread t owns positions t*KPT .. t*KPT+KPT-1 in every
// phase (its ids are loaded with independent loads, its outputs are KPT consecutive entries).  Ids are handled
// as 32-bit fields f = id - field_base (field_base = id_base for the 32-bit keys, 0 for the 64-bit ones; ids lie
// below 2^31): cluster bounds become wave-uniform 32-bit values from the kernel argument.
template <int KPT, typename KeyT>
__device__ __forceinline__ void embed_sort_body(
    const int64_t* __restrict__ ids, int n, int n_pow2, const EmbedClusterArgs& cl, int64_t id_base, int tok_bits, int radix_passes,
    int32_t* __restrict__ perm, int32_t* __restrict__ rows, int32_t* __restrict__ seg,
    int32_t* __restrict__ run_start, int64_t* __restrict__ uniq_ids, int32_t* __restrict__ run_id,
    KeyT* key, unsigned char* after_keys, SortShared& sh)
{
    constexpr KeyT kNone = ~(KeyT)0;
    constexpr bool kWide = sizeof(KeyT) == 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int e0 = tid * KPT;
    const int64_t field_base = kWide ? 0 : id_base;
    uint32_t flo[kEmbedMaxClusters], fhi[kEmbedMaxClusters];   // empty beyond the cluster count
#pragma unroll
    for (int q = 0; q < kEmbedMaxClusters; ++q) {
        flo[q] = q < cl.count ? (uint32_t)(cl.id_begin[q] - field_base) : 0u;
        fhi[q] = q < cl.count ? (uint32_t)(cl.id_end[q] - field_base) : 0u;
    }
    // (The whole block runs on one CU at one wave instruction per clock: its time is its instruction count,
    // about 50 per key and radix pass.)
    auto cluster_of_field = [&](uint32_t f, uint32_t& lo, uint32_t& hi) {
        int c = -1;
        lo = 0; hi = 0;
#pragma unroll
        for (int q = 0; q < kEmbedMaxClusters; ++q)
            if (f >= flo[q] && f < fhi[q]) { c = q; lo = flo[q]; hi = fhi[q]; }
        return c;
    };
    auto field_of = [&](KeyT kk) -> uint32_t { return kWide ? (uint32_t)((unsigned long long)kk >> 32) : (uint32_t)(kk >> tok_bits); };
    auto tok_of = [&](KeyT kk) -> int32_t {
        return kWide ? (int32_t)((unsigned long long)kk & 0xFFFFFFFFull) : (int32_t)(kk & (((KeyT)1 << tok_bits) - 1));
    };

    // keys: all loads of a thread are in flight together
    int64_t idv[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) idv[j] = (e0 + j < n) ? ids[e0 + j] : (int64_t)-1;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        KeyT kk = kNone;
        const int64_t rel = idv[j] - field_base;
        uint32_t lo, hi;
        if (e0 + j < n && rel >= 0 && rel < ((int64_t)1 << 32) && cluster_of_field((uint32_t)rel, lo, hi) >= 0)
            kk = kWide ? (KeyT)(((unsigned long long)(uint32_t)rel << 32) | (unsigned)(e0 + j))
                       : (KeyT)(((unsigned long long)(uint32_t)rel << tok_bits) | (unsigned)(e0 + j));
        key[e0 + j] = kk;
    }
    __syncthreads();

    if constexpr (!kWide) {
        // 32-bit keys: stable radix sort on the id field (radix_passes digits of 4 bits above the token bits)
        radix_sort_block<KPT>(key, (uint16_t*)after_keys, sh.wave_count, tok_bits, radix_passes);
    } else {
        // 64-bit keys: bitonic sorting network, ascending, on registers.  A stage pairs key e with key
        // e ^ stride: the partner lies in the same thread (stride < KPT), in the same wave (thread
        // t ^ stride/KPT, fetched with a lane shuffle) or in another wave (exchanged through LDS, two barriers).
        bitonic_sort_block<KPT, KeyT>(key, n_pow2);
    }

    // this thread's sorted keys and their two neighbours
    KeyT k[KPT + 2];
    k[0] = e0 > 0 ? key[e0 - 1] : kNone;
#pragma unroll
    for (int j = 0; j < KPT; ++j) k[j + 1] = key[e0 + j];
    k[KPT + 1] = e0 + KPT < n_pow2 ? key[e0 + KPT] : kNone;

    // per-position outputs, cluster segments, run heads
    int heads = 0;
    unsigned head_mask = 0;
    int c = -1;
    uint32_t c_lo = 0, c_hi = 0;
    constexpr int G = KPT % 4 == 0 ? 4 : 1;   // outputs leave 16 bytes at a time where four positions exist
#pragma unroll
    for (int q = 0; q < KPT / G; ++q) {
        int32_t perm_v[G], rows_v[G];   // positions without a token (sorted last, never read) get 0
#pragma unroll
        for (int e = 0; e < G; ++e) {
            const int j = q * G + e;
            const KeyT kj = k[j + 1];
            perm_v[e] = 0; rows_v[e] = 0;
            if (kj == kNone) continue;
            const int i = e0 + j;
            const uint32_t f = field_of(kj);
            if (!(c >= 0 && f >= c_lo && f < c_hi)) c = cluster_of_field(f, c_lo, c_hi);   // sorted: rarely changes
            perm_v[e] = tok_of(kj);
            rows_v[e] = (int32_t)(f - c_lo);
            // sorted ids: a neighbour belongs to another cluster iff it falls outside this one's range
            const bool has_prev = i > 0, has_next = k[j + 2] != kNone;
            if (!has_prev || field_of(k[j]) < c_lo) sh.first[c] = i;
            if (!has_next || field_of(k[j + 2]) >= c_hi) sh.last[c] = i + 1;
            if (!has_next) sh.valid = i + 1;
            if (!has_prev || field_of(k[j]) != f) { head_mask |= 1u << j; ++heads; }
        }
        const int i0 = e0 + q * G;
        if constexpr (G == 4) {
            if (i0 + 3 < n) {
                *(i32x4*)(perm + i0) = i32x4{perm_v[0], perm_v[1], perm_v[2], perm_v[3]};
                *(i32x4*)(rows + i0) = i32x4{rows_v[0], rows_v[1], rows_v[2], rows_v[3]};
                continue;
            }
        }
#pragma unroll
        for (int e = 0; e < G; ++e)
            if (i0 + e < n) { perm[i0 + e] = perm_v[e]; rows[i0 + e] = rows_v[e]; }
    }
    // runs of equal ids: block-wide exclusive scan of the head counts
    const int incl = wave_inclusive_scan(heads);
    if (lane == 63) sh.wave_count[wave] = incl;
    // this barrier orders LDS traffic only; it does not wait for the global stores above
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    int u = incl - heads, total = 0;
#pragma unroll
    for (int wv = 0; wv < kSortThreads / 64; ++wv) {
        const int wc = sh.wave_count[wv];
        u += wv < wave ? wc : 0;
        total += wc;
    }
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const KeyT kj = k[j + 1];
        if (kj == kNone) continue;
        const int i = e0 + j;
        if (head_mask & (1u << j)) {
            run_start[u] = i;
            uniq_ids[u] = (int64_t)field_of(kj) + field_base;
            ++u;
        }
        run_id[i] = u - 1;   // the run that holds sorted position i
    }
    if (tid < kEmbedMaxClusters) {
        seg[2 * tid] = (tid < cl.count) ? sh.first[tid] : 0;
        seg[2 * tid + 1] = (tid < cl.count) ? sh.last[tid] - sh.first[tid] : 0;
    }
    if (tid == 0) {
        run_start[total] = sh.valid;
        seg[kSegUnique] = total;
        seg[kSegValid] = sh.valid;
    }
}

// One block.  Outputs: perm[i] = token at sorted position i, rows[i] = its row in
// the cluster's table, seg (see above), run_start[u] = first sorted position of
// the u-th distinct id (run_start[n_unique] = number of valid tokens),
// uniq_ids[u] = that id, run_id[i] = index u of the run that holds sorted position i.  Ids outside every cluster sort last and are ignored.
// Keys: id and token position packed so that equal ids keep token order.  KeyT = 64 bits:
// id << 32 | token.  KeyT = 32 bits, when (largest id - id_base) and the token positions fit
// together: (id - id_base) << tok_bits | token, sorted by a stable radix sort on the id field.
// KPT = n_pow2 / kSortThreads keys per thread (1, 2, 4, 8 or 16): a kernel per value, so that the registers of a
// small batch are not those of the largest.
template <typename KeyT, int KPT>
__global__ __launch_bounds__(kSortThreads) void embed_sort_kernel(
    const int64_t* __restrict__ ids, int n, int n_pow2, EmbedClusterArgs cl, int64_t id_base, int tok_bits, int radix_passes,
    int32_t* __restrict__ perm, int32_t* __restrict__ rows, int32_t* __restrict__ seg,
    int32_t* __restrict__ run_start, int64_t* __restrict__ uniq_ids, int32_t* __restrict__ run_id)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    __shared__ SortShared sh;
    const int tid = threadIdx.x;
    if (tid < kEmbedMaxClusters) { sh.first[tid] = 0; sh.last[tid] = 0; }
    if (tid == 0) sh.valid = 0;
    __syncthreads();
    KeyT* key = (KeyT*)smem_raw;
    unsigned char* after_keys = smem_raw + (size_t)n_pow2 * sizeof(KeyT);
    embed_sort_body<KPT, KeyT>(ids, n, n_pow2, cl, id_base, tok_bits, radix_passes, perm, rows, seg, run_start,
                               uniq_ids, run_id, key, after_keys, sh);
}

// g_c[i - first_c, :] = round(E_c[rows[i], :] .* z_c), one block per sorted position.
template <int ES>
__global__ __launch_bounds__(128) void embed_gather_gate_kernel(
    EmbedClusterArgs cl, const int32_t* __restrict__ rows, const int32_t* __restrict__ seg)
{
    const int i = blockIdx.x;
    // a kernel starts with cold caches, so every dependent load costs a trip to memory: the row number is requested
    // together with the segment table (the sort writes rows[] for every position, 0 where there is no token)
    const int row = rows[i];
    if (i >= seg[kSegValid]) return;
    const int c = cluster_at(seg, cl.count, i);
    if (c < 0) return;
    const int dim = cl.dim[c];
    const char* src = (const char*)cl.E[c] + (int64_t)row * cl.lde[c] * ES;
    char* dst = (char*)cl.g[c] + (int64_t)(i - seg[2 * c]) * cl.ldg[c] * ES;
    const float* z = cl.z[c];
    int k0 = 0;
    if (ES == 2 && (((uintptr_t)src | (uintptr_t)dst) & 15u) == 0) {
        // 8 bfloat16 at a time while whole 16-byte chunks remain (rows start 16-byte aligned)
        for (int k = threadIdx.x * 8; k + 8 <= dim; k += 128 * 8) {
            const u32x4 e = *(const u32x4*)(src + k * 2);
            u32x4 o;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float lo = __builtin_bit_cast(float, e[w] << 16) * z[k + 2 * w];
                const float hi = __builtin_bit_cast(float, e[w] & 0xFFFF0000u) * z[k + 2 * w + 1];
                o[w] = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)lo) | ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)hi) << 16);
            }
            *(u32x4*)(dst + k * 2) = o;
        }
        k0 = dim & ~7;
    }
    for (int k = k0 + threadIdx.x; k < dim; k += 128) {
        if (ES == 2) {
            const float e = __builtin_bit_cast(float, (uint32_t)((const uint16_t*)src)[k] << 16);
            ((uint16_t*)dst)[k] = __builtin_bit_cast(uint16_t, (__bf16)(e * z[k]));
        } else {
            ((float*)dst)[k] = ((const float*)src)[k] * z[k];
        }
    }
}

// dst[i, :] = src[perm[i], :] for the valid sorted positions; 16-byte copies when allowed.
template <int ES>
__global__ __launch_bounds__(kStreamThreads) void gather_rows_kernel(
    const void* __restrict__ src, int64_t lds_, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ seg, int cols, void* __restrict__ dst, int64_t ldd, int vec_ok)
{
    const int i = blockIdx.x;
    if (i >= seg[kSegValid]) return;
    const char* s = (const char*)src + (int64_t)perm[i] * lds_ * ES;
    char* d = (char*)dst + (int64_t)i * ldd * ES;
    const int64_t bytes = (int64_t)cols * ES;
    if (vec_ok) {
        for (int64_t b = (int64_t)threadIdx.x * 16; b + 16 <= bytes; b += (int64_t)kStreamThreads * 16)
            *(uint4*)(d + b) = *(const uint4*)(s + b);
        const int64_t tail = bytes & ~(int64_t)15;
        for (int64_t b = tail + threadIdx.x * ES; b < bytes; b += (int64_t)kStreamThreads * ES)
            for (int e = 0; e < ES; ++e) d[b + e] = s[b + e];
    } else {
        for (int64_t b = (int64_t)threadIdx.x * ES; b < bytes; b += (int64_t)kStreamThreads * ES)
            for (int e = 0; e < ES; ++e) d[b + e] = s[b + e];
    }
}

// ---- embedding gradient: dE_c[row, :] = sum over the run of equal ids of dh_c[i - first_c, :] ----
// Runs are contiguous in sorted order but very uneven (a frequent word can own a
// tenth of the batch), so the sorted positions are cut into windows of
// kScatterWindow rows, one block each.  A run that lies inside one window is
// summed and stored there.  A run that crosses window borders leaves float32
// partial sums: `tail` in the window where it starts, `head` in every later
// window it reaches; a second kernel adds them in window order.  Float32
// accumulation in a fixed order and one rounding: deterministic.
constexpr int kScatterWindow = 32;
constexpr int kScatterThreads = 256;

template <int ES>
__device__ __forceinline__ float load_elem(const char* p, int64_t idx)
{
    if (ES == 2) return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)p)[idx] << 16);
    return ((const float*)p)[idx];
}

template <int ES>
__device__ __forceinline__ void store_elem(char* p, int64_t idx, float v)
{
    if (ES == 2) ((uint16_t*)p)[idx] = __builtin_bit_cast(uint16_t, (__bf16)v);
    else ((float*)p)[idx] = v;
}

// head, tail: [windows][ldp] floats.  Block (w, cb) handles window w and the columns
// cb*256 .. cb*256+255.  Threads 0..31 describe the window's rows (source row, width, and where
// the sum goes if the row ends a run or the window); then every thread owns one column, loads it
// for all rows at once and adds in row order.
template <int ES>
__global__ __launch_bounds__(kScatterThreads) void embed_scatter_window_kernel(
    EmbedClusterArgs cl, const int32_t* __restrict__ rows, const int32_t* __restrict__ seg,
    const int32_t* __restrict__ run_start, const int32_t* __restrict__ run_id,
    float* __restrict__ head, float* __restrict__ tail, int64_t ldp, int n)
{
    __shared__ const char* row_src[kScatterWindow];
    __shared__ char* row_dst[kScatterWindow];
    __shared__ int row_dim[kScatterWindow];    // 0: row not used
    __shared__ int row_flush[kScatterWindow];  // 0: keep adding, 1: round and store to dE, 2: store float32 partial
    const int w0 = blockIdx.x * kScatterWindow;   // < n: the grid has ceil(n / window) windows
    // A kernel starts with cold caches, so every dependent load costs a trip to memory.  What depends on the position
    // alone is requested before the batch's extents are known: the run and the table row of this thread's position
    // (rows[] is written for all n positions; run_id[] beyond the valid ones holds anything and is not used).
    int u = 0, row = 0;
    if (threadIdx.x < kScatterWindow) {
        const int ic = min(w0 + (int)threadIdx.x, n - 1);
        u = run_id[ic];
        row = rows[ic];
    }
    const int valid = seg[kSegValid];
    if (w0 >= valid) return;
    const int w1 = (w0 + kScatterWindow < valid) ? w0 + kScatterWindow : valid;
    // Rows of the window first (they depend on the segment table only), so that their loads below and the run
    // extents travel together.
    int c = -1, r0 = 0, r1 = 0;
    if (threadIdx.x < kScatterWindow) {
        const int t = threadIdx.x, i = w0 + t;
        row_dim[t] = 0; row_flush[t] = 0; row_src[t] = nullptr; row_dst[t] = nullptr;
        if (i < w1) {
            c = cluster_at(seg, cl.count, i);   // a run lies inside one cluster
            if (c >= 0 && cl.dE[c]) {
                row_dim[t] = cl.dim[c];
                row_src[t] = (const char*)cl.g[c] + (int64_t)(i - seg[2 * c]) * cl.ldg[c] * ES;
                r0 = run_start[u];
                r1 = run_start[u + 1];
            } else {
                c = -1;
            }
        }
    }
    __syncthreads();
    const int k = blockIdx.y * kScatterThreads + threadIdx.x;
    float v[kScatterWindow];
#pragma unroll
    for (int t = 0; t < kScatterWindow; ++t) v[t] = (k < row_dim[t]) ? load_elem<ES>(row_src[t], k) : 0.0f;
    if (threadIdx.x < kScatterWindow && c >= 0) {
        const int t = threadIdx.x, i = w0 + t;
        const int end = (r1 < w1) ? r1 : w1;
        if (i == end - 1) {
            if (r0 >= w0 && r1 <= w1) {
                row_flush[t] = 1;
                row_dst[t] = (char*)cl.dE[c] + (int64_t)row * cl.ldde[c] * ES;   // every position of a run has its row
            } else {
                row_flush[t] = 2;
                row_dst[t] = (char*)(((r0 < w0) ? head : tail) + (int64_t)blockIdx.x * ldp);
            }
        }
    }
    __syncthreads();
    float acc = 0.0f;
#pragma unroll
    for (int t = 0; t < kScatterWindow; ++t) {
        acc += v[t];
        const int fl = row_flush[t];
        if (fl != 0) {
            if (k < row_dim[t]) {
                if (fl == 1) store_elem<ES>(row_dst[t], k, acc);
                else ((float*)row_dst[t])[k] = acc;
            }
            acc = 0.0f;
        }
    }
}

template <int ES>
__global__ __launch_bounds__(kScatterThreads) void embed_scatter_join_kernel(
    EmbedClusterArgs cl, const int32_t* __restrict__ rows, const int32_t* __restrict__ seg,
    const int32_t* __restrict__ run_start, const int32_t* __restrict__ run_id, const float* __restrict__ head,
    const float* __restrict__ tail, int64_t ldp, int n)
{
    const int w0 = blockIdx.x * kScatterWindow;   // < n
    // the window's last position, requested before the batch's extents are known (see the window kernel); only the
    // batch's last window ends earlier and asks again
    const int ic = min(w0 + kScatterWindow - 1, n - 1);
    int u = run_id[ic], row = rows[ic];
    const int valid = seg[kSegValid];
    if (w0 >= valid) return;
    const int w1 = (w0 + kScatterWindow < valid) ? w0 + kScatterWindow : valid;
    if (w1 - 1 != ic) { u = run_id[w1 - 1]; row = rows[w1 - 1]; }
    // the run that leaves this window through its end, if it also starts here
    const int r0 = run_start[u], r1 = run_start[u + 1];
    if (r0 < w0 || r1 <= w1) return;
    const int c = cluster_at(seg, cl.count, r0);
    if (c < 0 || !cl.dE[c]) return;
    const int last = (r1 - 1) / kScatterWindow;
    const int dim = cl.dim[c];
    char* dst = (char*)cl.dE[c] + (int64_t)row * cl.ldde[c] * ES;
    for (int k = threadIdx.x; k < dim; k += kScatterThreads) {
        float acc = tail[(int64_t)blockIdx.x * ldp + k];
#pragma unroll 8
        for (int b = (int)blockIdx.x + 1; b <= last; ++b) acc += head[(int64_t)b * ldp + k];
        store_elem<ES>(dst, k, acc);
    }
}

__global__ void embed_touched_kernel(const int64_t* __restrict__ uniq_ids, const int32_t* __restrict__ seg,
                                     int64_t* __restrict__ touched_ids, int32_t* __restrict__ n_touched)
{
    const int nu = seg[kSegUnique];
    if (n_touched && blockIdx.x == 0 && threadIdx.x == 0) n_touched[0] = nu;
    if (touched_ids)
        for (int u = blockIdx.x * blockDim.x + threadIdx.x; u < nu; u += gridDim.x * blockDim.x)
            touched_ids[u] = uniq_ids[u];
}

}  // namespace flop
