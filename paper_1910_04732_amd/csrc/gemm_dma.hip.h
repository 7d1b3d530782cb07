// bfloat16 contraction kernel with asynchronous global -> LDS staging (gfx950).
//
// Same grouped-problem interface and epilogue as gemm_tile.hip.h, for operands
// that allow 16-byte transfers (16-byte aligned bases, leading dimensions that
// are multiples of 8 elements; the last 16-byte chunk of a row may reach into
// the row's padding).  Differences:
//   * tiles go from global memory straight into LDS with
//     buffer_load_dwordx4 ... lds (no register staging), NSTAGE steps of 64 k
//     deep, so that several steps of memory latency are in flight while the
//     matrix cores work; the buffer descriptor's range check zero-fills rows
//     beyond the matrix, explicit out-of-range offsets zero-fill the k tail
//     (elements beyond a K that is not a multiple of 8 are cleared in LDS);
//   * an operand whose contiguous dimension is k is stored [row][k] with the
//     16-byte chunks of a row XOR-swizzled by the row index (conflict-free
//     ds_read_b128 fragment reads);
//   * an operand whose contiguous dimension is the row index (the transposed
//     products dy^T g, dh^T x and the right-hand sides dy P, dh Q) is stored as
//     it lies in memory, [k][row], with 64-byte segments XOR-swizzled by k, and
//     is fetched with ds_read_b64_tr_b16, which transposes 4x16 blocks on the
//     way into the MFMA operand layout;
//   * blocks map to tiles through locate_tile(): each XCD works on a contiguous
//     range of every product's tiles and re-uses panels in its own L2;
//   * a block is G groups of WM x WN wavefronts.  Every group covers the whole
//     BM x BN tile (a wavefront owns a (BM/WM) x (BN/WN) part of it) but only
//     every G-th 64-k step of the contraction, with stage buffers, transfers
//     and accumulators of its own; the groups' sums are added through LDS before
//     the epilogue.  A launch with few tiles per compute unit then has G times
//     the bytes in flight per tile and G wavefronts per SIMD, and a tile takes
//     1/G of the steps (the groups share the block's barriers: all take the
//     same number of steps, a step beyond K is zero-filled).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "gemm_tile.hip.h"

namespace flop {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#ifndef FLOP_LDS_PTR   // a host build of the address arithmetic defines its own
#define FLOP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#endif

// s_waitcnt that waits only for vmcnt <= N (lgkmcnt / expcnt left alone).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

constexpr uint32_t kOutOfRange = 0x80000000u;   // beyond any descriptor we build (ranges < 2 GiB)
constexpr int kKtabMaxK = 4096;                 // longest contraction over gathered k rows
constexpr int kKtabBytes = (kKtabMaxK + 256) * 2;   // its table in LDS: 16-bit row numbers, rounded up to a step of 4 groups
constexpr uint32_t kKtabNone = 0xFFFFu;         // table entry of a k beyond the contraction

template <typename SH>
constexpr size_t gemm_dma_lds_bytes();

// Swizzle of a [k][row] stage with S 64-byte segments per k row: segment index seg of k row krow is stored at
// segment kr_swizzle<S>(krow, seg).  Four consecutive k rows (what one transposing fragment read touches per
// 16 lanes) must land in four different 64-byte bank groups: with a row pitch of 128, 256 or 512 bytes the
// segment is XOR-ed with bits of the k row; with 64 or 192 bytes consecutive rows already do.
template <int S>
__device__ __forceinline__ int kr_swizzle(int krow, int seg)
{
    static_assert(S == 1 || S == 2 || S == 3 || S == 4 || S == 8, "stage rows per operand: 32, 64, 96, 128 or 256");
    if constexpr (S == 2) return seg ^ ((krow >> 1) & 1);
    else if constexpr (S == 4 || S == 8) return seg ^ (krow & 3);
    else return seg;
}

// Per-thread transfer plan of one operand stage: ROWS rows (m or n) by 64 k, filled by the NW wavefronts of a
// group (ROWS a multiple of 8 NW: a wave instruction fills 64 slots of 16 bytes).  The group contracts the
// k ranges [64 (s G + g), +64), s = 0 .. nk - 1.
template <int ROWS, int NW>
struct DmaPlan {
    static_assert(ROWS % (8 * NW) == 0, "stage rows must divide among the group's wavefronts");
    static constexpr int NV = ROWS / (8 * NW);    // 16-byte transfers per thread and step
    uint32_t voff[NV];       // byte offset of each transfer at step 0 (kOutOfRange: zero-fill)
    uint32_t tail_bit[NV];   // kOutOfRange where the transfer lies beyond K in the group's last step
    uint32_t step_bytes;     // added per step (scalar offset)
    // A [k][row] operand whose k rows are gathered through an index list: ktab (LDS) holds the matrix row of
    // every k of the contraction (kKtabNone beyond K), voff only the column part, kidx[p] the transfer's k
    // at step 0, and kv[p] the byte offsets of the rows of the step that is issued next, read one step ahead.
    const uint16_t* ktab;    // nullptr: not gathered
    uint32_t kidx[NV], kv[NV], kstep, row_bytes;

    // kmajor: X[row*ld + k]      otherwise: X[k*ld + row]
    // tid: thread index inside the group; k_first: first k of the group (64 g); k_stride: 64 G; nk: steps
    // map (nullable): rows (kmajor) are rows map[row] of the matrix; ktab_ (nullable, !kmajor): see ktab
    __device__ __forceinline__ void init(int kmajor, int64_t ld, int row0, int rows, int K, int tid, int k_first,
                                         int k_stride, int nk, const int32_t* map = nullptr, const uint16_t* ktab_ = nullptr)
    {
        ktab = kmajor ? nullptr : ktab_;
        kstep = (uint32_t)k_stride;
        row_bytes = (uint32_t)(ld * 2);
        const int wave = tid >> 6, lane = tid & 63;
        const int ktail0 = (nk - 1) * k_stride + k_first;   // first k of the group's last step
#pragma unroll
        for (int p = 0; p < NV; ++p) {
            const int pos = (p * NW + wave) * 64 + lane;   // 16-byte slot inside the stage buffer
            if (kmajor) {
                const int row = pos >> 3, cp = pos & 7;
                const int c = cp ^ ((row >> 1) & 7);
                const bool inside = row0 + row < rows;
                const int64_t src_row = (map && inside) ? map[row0 + row] : row0 + row;
                voff[p] = inside ? (uint32_t)((src_row * ld + k_first + c * 8) * 2) : kOutOfRange;
                tail_bit[p] = (ktail0 + c * 8 < K) ? 0u : kOutOfRange;
                kidx[p] = 0; kv[p] = 0;
            } else {
                constexpr int CPR = ROWS / 8;             // 16-byte chunks per k-row
                constexpr int S = ROWS / 32;              // 64-byte segments per k-row
                const int krow = pos / CPR, cc = pos % CPR;
                // the slot at stored segment cc / 4 holds the source segment that the swizzle maps there
                int src_seg = cc >> 2;
                if constexpr (S == 2 || S == 4 || S == 8) src_seg = kr_swizzle<S>(krow, cc >> 2);   // XOR: its own inverse
                const int m = row0 + src_seg * 32 + (cc & 3) * 8;
                if (ktab) voff[p] = (m < rows) ? (uint32_t)(m * 2) : kOutOfRange;
                else voff[p] = (m < rows) ? (uint32_t)(((int64_t)(k_first + krow) * ld + m) * 2) : kOutOfRange;
                tail_bit[p] = 0u;                         // k rows beyond K fail the range check
                kidx[p] = (uint32_t)(k_first + krow);
                kv[p] = 0;
            }
        }
        step_bytes = kmajor ? (uint32_t)(k_stride * 2) : (uint32_t)((int64_t)k_stride * ld * 2);
        if (ktab) step_bytes = 0;
    }

    // gathered k rows: read the table entries of `step` (the next one to be issued)
    __device__ __forceinline__ void fetch_k(int step)
    {
        if (!ktab) return;
#pragma unroll
        for (int p = 0; p < NV; ++p) {
            const uint32_t row = ktab[(uint32_t)step * kstep + kidx[p]];
            kv[p] = row == kKtabNone ? kOutOfRange : row * row_bytes;
        }
    }

    // Pins the table entries read by fetch_k into registers here: call right after the wait that drains the
    // wave's LDS reads, so that the compiler's own wait for them lands there and not among the fragment reads.
    __device__ __forceinline__ void settle_k()
    {
        if (!ktab) return;
#pragma unroll
        for (int p = 0; p < NV; ++p) asm volatile("" : "+v"(kv[p]));
    }

    // byte offset of transfer p: the plan's own, or column part + the k row's table entry (either may be out of range)
    __device__ __forceinline__ uint32_t offset_of(int p, uint32_t tail_mask) const
    {
        const uint32_t own = voff[p] | (tail_bit[p] & tail_mask);
        if (!ktab) return own;
        return (own + kv[p]) | ((own | kv[p]) & kOutOfRange);
    }

    // transfer number p of the plan alone (p is a compile-time constant at every call site)
    __device__ __forceinline__ void issue_one(int p, __amdgpu_buffer_rsrc_t rsrc, unsigned char* stage, int step,
                                              uint32_t tail_mask, int wave) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FLOP_LDS_PTR(stage + (p * NW + wave) * 1024), 16,
                                                 offset_of(p, tail_mask), (uint32_t)step * step_bytes, 0, 0);
    }

    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, unsigned char* stage, int step,
                                          uint32_t tail_mask, int wave) const
    {
        const uint32_t soff = (uint32_t)step * step_bytes;
#pragma unroll
        for (int p = 0; p < NV; ++p)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FLOP_LDS_PTR(stage + (p * NW + wave) * 1024), 16,
                                                     offset_of(p, tail_mask), soff, 0, 0);
    }
};

// The same stage layout filled with 4-byte transfers, for operands whose rows are only
// 4-byte aligned (even leading dimension, e.g. unpadded 410-wide matrices).  A wave
// instruction fills 256 consecutive LDS bytes = 16 chunk slots; lane / 4 picks the slot,
// lane % 4 the dword inside it.  Transfer p of a lane differs from transfer 0 only by a
// wave-uniform row offset (and, for [row][k], by which of two swizzled chunks it reads), so
// the plan is a handful of registers.  Rows beyond the matrix need no test: their offsets
// lie beyond the descriptor's range and are zero-filled.
template <int ROWS>
struct DmaPlan4 {
    static constexpr int NV = ROWS / 8;           // 4-byte transfers per thread and step
    uint32_t voff2[2];       // offsets for even / odd p (they differ in the chunk swizzle of [row][k])
    uint32_t tail2[2];       // kOutOfRange where the dword lies beyond K in a partial last step
    uint32_t p_bytes;        // added per transfer index p (scalar)
    uint32_t step_bytes;

    // same signature as DmaPlan::init; only used by blocks of one group (k_first = 0, k_stride = 64)
    // (gathered operands are never routed to 4-byte transfers: the last two arguments are ignored)
    __device__ __forceinline__ void init(int kmajor, int64_t ld, int row0, int rows, int K, int tid, int /*k_first*/,
                                         int /*k_stride*/, int nk, const int32_t* = nullptr, const uint16_t* = nullptr)
    {
        const int wave = tid >> 6, lane = tid & 63;
        const int ktail0 = (nk - 1) * 64;
        const int w = lane & 3;
        if (kmajor) {
            // slot = (4p + wave) * 16 + lane / 4: row = (4p + wave) * 2 + lane / 32, chunk position (lane / 4) % 8
            const int cp = (lane >> 2) & 7;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int row = (4 * q + wave) * 2 + (lane >> 5);
                const int c = cp ^ ((row >> 1) & 7);
                voff2[q] = (uint32_t)(((int64_t)(row0 + row) * ld + c * 8 + w * 2) * 2) - (uint32_t)q * (uint32_t)(8 * ld * 2);
                tail2[q] = (ktail0 + c * 8 + w * 2 < K) ? 0u : kOutOfRange;
            }
            p_bytes = (uint32_t)(8 * ld * 2);      // 8 rows per p
            step_bytes = 128u;
        } else {
            constexpr int CPR = ROWS / 8, S = ROWS / 32;
            const int slot = wave * 16 + (lane >> 2);
            const int krow = slot / CPR, cc = slot % CPR;      // p adds 64 / CPR k-rows, which leaves the swizzle alone
            const int f = (S == 2) ? ((krow >> 1) & 1) : (krow & 3);
            const int seg = (cc >> 2) ^ f;
            const int m = row0 + seg * 32 + (cc & 3) * 8 + w * 2;
            voff2[0] = voff2[1] = (m < rows) ? (uint32_t)(((int64_t)krow * ld + m) * 2) : kOutOfRange;
            tail2[0] = tail2[1] = 0u;
            p_bytes = (uint32_t)((64 / CPR) * ld * 2);
            step_bytes = (uint32_t)(64 * ld * 2);
        }
    }

    __device__ __forceinline__ void issue_one(int p, __amdgpu_buffer_rsrc_t rsrc, unsigned char* stage, int step,
                                              uint32_t tail_mask, int wave) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FLOP_LDS_PTR(stage + (p * 4 + wave) * 256), 4,
                                                 voff2[p & 1] | (tail2[p & 1] & tail_mask),
                                                 (uint32_t)step * step_bytes + (uint32_t)p * p_bytes, 0, 0);
    }

    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, unsigned char* stage, int step,
                                          uint32_t tail_mask, int wave) const
    {
#pragma unroll
        for (int p = 0; p < NV; ++p) issue_one(p, rsrc, stage, step, tail_mask, wave);
    }
    __device__ __forceinline__ void fetch_k(int) {}
    __device__ __forceinline__ void settle_k() {}
};

// One MFMA operand fragment: 8 bfloat16 (k = 16*kc + 8*(lane/32) + 0..7) of row lane%32,
// filled either by one 16-byte read (q) or by two transposing 8-byte reads (h).
union Frag {
    u32x4 q;
    u32x2 h[2];
    __device__ __forceinline__ bf16x8 get() const { return __builtin_bit_cast(bf16x8, q); }
};

// Fragment addressing of one operand for one wave: T 32-row MFMA tiles of a
// ROWS-row stage buffer.  KMAJOR: [row][k] swizzled chunks, one 16-byte read.
// Otherwise [k][row] with swizzled 64-byte segments, two transposing reads
// issued from inline assembly (the caller waits on lgkmcnt before use).
template <int ROWS, int T, bool KMAJOR>
struct FragReader {
    uint32_t base[T];   // per-lane byte offset inside a stage buffer, per MFMA tile
    uint32_t x;         // k-major: lane part of the chunk swizzle

    __device__ __forceinline__ void init(int wave_row0, int lane)
    {
        const int l32 = lane & 31, lhi = lane >> 5;
        if constexpr (KMAJOR) {
            x = (uint32_t)(lhi ^ ((l32 >> 1) & 7));
#pragma unroll
            for (int t = 0; t < T; ++t) base[t] = (uint32_t)((wave_row0 + t * 32 + l32) * 128);
        } else {
            constexpr int S = ROWS / 32;
            const int kr = (lane >> 2) & 3;             // k row this lane fetches for the 4x16 transpose
            x = 0;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int m = wave_row0 + t * 32 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
                const int seg = kr_swizzle<S>(kr, m >> 5);
                base[t] = (uint32_t)((lhi * 8 + kr) * (ROWS * 2) + seg * 64 + (m & 31) * 2);
            }
        }
    }

    template <int KC>
    __device__ __forceinline__ void load(uint32_t stage_lds_addr, int t, Frag& f) const
    {
        if constexpr (KMAJOR) {
            const uint32_t addr = stage_lds_addr + base[t] + (((uint32_t)(KC << 1) ^ x) << 4);
            asm volatile("ds_read_b128 %0, %1" : "=v"(f.q) : "v"(addr));
        } else {
            const uint32_t addr = stage_lds_addr + base[t];
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.h[0]) : "v"(addr), "n"(KC * 16 * ROWS * 2));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                         : "=v"(f.h[1]) : "v"(addr), "n"(KC * 16 * ROWS * 2 + 4 * ROWS * 2));
        }
    }
};

// All fragments of one 64-k step for one wave: 4 chunks of 16 k.
template <int TM, int TN>
struct FragSet {
    Frag a[4][TM], b[4][TN];
};

// Wait for every LDS read this wave has issued.  The fragments about to be
// consumed are read-write operands of the statement, so their consumers cannot
// be scheduled ahead of the wait.
template <int TM, int TN>
__device__ __forceinline__ void wait_fragset(FragSet<TM, TN>& f)
{
    static_assert(TM <= 2 && TN <= 2, "extend the operand list");
#define FLOP_FA(k, i) "+v"(f.a[k][i].q)
#define FLOP_FB(k, j) "+v"(f.b[k][j].q)
    if constexpr (TM == 2 && TN == 2)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : FLOP_FA(0, 0), FLOP_FA(0, 1), FLOP_FA(1, 0), FLOP_FA(1, 1), FLOP_FA(2, 0), FLOP_FA(2, 1),
                       FLOP_FA(3, 0), FLOP_FA(3, 1), FLOP_FB(0, 0), FLOP_FB(0, 1), FLOP_FB(1, 0), FLOP_FB(1, 1),
                       FLOP_FB(2, 0), FLOP_FB(2, 1), FLOP_FB(3, 0), FLOP_FB(3, 1));
    else if constexpr (TM == 2 && TN == 1)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : FLOP_FA(0, 0), FLOP_FA(0, 1), FLOP_FA(1, 0), FLOP_FA(1, 1), FLOP_FA(2, 0), FLOP_FA(2, 1),
                       FLOP_FA(3, 0), FLOP_FA(3, 1), FLOP_FB(0, 0), FLOP_FB(1, 0), FLOP_FB(2, 0), FLOP_FB(3, 0));
    else if constexpr (TM == 1 && TN == 2)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : FLOP_FA(0, 0), FLOP_FA(1, 0), FLOP_FA(2, 0), FLOP_FA(3, 0), FLOP_FB(0, 0), FLOP_FB(0, 1),
                       FLOP_FB(1, 0), FLOP_FB(1, 1), FLOP_FB(2, 0), FLOP_FB(2, 1), FLOP_FB(3, 0), FLOP_FB(3, 1));
    else
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : FLOP_FA(0, 0), FLOP_FA(1, 0), FLOP_FA(2, 0), FLOP_FA(3, 0), FLOP_FB(0, 0), FLOP_FB(1, 0),
                       FLOP_FB(2, 0), FLOP_FB(3, 0));
#undef FLOP_FA
#undef FLOP_FB
}

// Shape of a block: BM x BN output tile, NB stage buffers per group, WM x WN wavefronts per group, G groups
// that take the 64-k steps of the contraction in turn.
template <int BM_, int BN_, int NB_, int WM_, int WN_, int G_>
struct TileShape {
    static constexpr int BM = BM_, BN = BN_, NB = NB_, WM = WM_, WN = WN_, G = G_;
    static constexpr int NWG = WM * WN;                 // wavefronts per group
    static constexpr int THREADS = 64 * NWG * G;
    static constexpr int WTM = BM / WM, WTN = BN / WN;  // a wavefront's part of the tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;  // in 32x32 MFMA tiles
    // stage rows: the tile's, rounded up so that the group's wavefronts fill them with whole instructions
    static constexpr int round_rows(int rows) { return (rows + 8 * NWG - 1) / (8 * NWG) * (8 * NWG); }
    static constexpr int AR = round_rows(BM), BR = round_rows(BN);
    static constexpr int A_BYTES = AR * 128, B_BYTES = BR * 128, STAGE = A_BYTES + B_BYTES;
    static constexpr int GROUP_BYTES = NB * STAGE;
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && TM >= 1 && TN >= 1 && TM <= 2 && TN <= 2, "wave tile");
    static_assert(THREADS <= 1024 && G >= 1, "block size");
    static_assert(AR % 32 == 0 && BR % 32 == 0, "stage rows are whole 64-byte segments of a [k][row] stage");
    static_assert(THREADS % (BN / 8) == 0, "the epilogue hands whole tile rows to the block's threads");
};

// Main loop of one group of wavefronts over its share of the k steps.  NB stage buffers in LDS are filled by
// asynchronous transfers; the fragments of step s+1 are read from LDS into a
// second register set while the matrix cores consume the set of step s, so
// that transfers, LDS reads and MFMAs of neighbouring steps overlap:
//   iteration s:  wait(reads of s) ; wait(transfers of s+1) ; barrier ;
//                 issue transfers of s+NB ; issue reads of s+1 ; MFMAs of s
// The barriers are the block's: every group executes the same sequence of them.
template <typename SH, bool AKM, bool BKM, int XFER = 16>
struct DmaLoop {
    static constexpr int BM = SH::BM, BN = SH::BN, NB = SH::NB, TM = SH::TM, TN = SH::TN;
    static constexpr int A_BYTES = SH::A_BYTES, STAGE = SH::STAGE;
    static_assert(XFER == 16 || XFER == 4, "transfer width");
    static_assert(XFER == 16 || (SH::NWG == 4 && SH::G == 1 && SH::AR == BM && SH::BR == BN), "4-byte transfers: one group of four");
    using PlanA = std::conditional_t<XFER == 16, DmaPlan<SH::AR, SH::NWG>, DmaPlan4<BM>>;
    using PlanB = std::conditional_t<XFER == 16, DmaPlan<SH::BR, SH::NWG>, DmaPlan4<BN>>;
    static constexpr int LPS = PlanA::NV + PlanB::NV;   // transfers per thread and stage
    static_assert(NB >= 2 && NB <= 6 && (NB - 1) * LPS < 64, "vmcnt budget");

    __amdgpu_buffer_rsrc_t ra, rb;
    PlanA pa;
    PlanB pb;
    FragReader<SH::AR, TM, AKM> fa;
    FragReader<SH::BR, TN, BKM> fb;
    unsigned char* smem;    // the group's stage buffers
    uint32_t smem_addr;
    int nk, wave;           // steps of every group; wavefront index inside the group
    bool ktail;
    int kfix, kfix_chunk;   // K % 8 (elements of the chunk that straddles K); that chunk's index in this group's last
                            // step, or -1 if it lies in another group's

    // group: index of this wavefront's group; smem_: start of the block's dynamic LDS; ktab: the table of k-row
    // offsets in LDS when B is a [k][row] operand gathered by pr.b_map (filled by the caller), else nullptr
    __device__ __forceinline__ void init(const GemmProblem& pr, unsigned char* smem_, int m0, int n0, int group,
                                         const uint16_t* ktab)
    {
        const int tid = threadIdx.x % (64 * SH::NWG);
        const int lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS targets of the transfers scalar
        const int wm = wave / SH::WN, wn = wave % SH::WN;
        // whole transfers: the last 16-byte chunk (4-byte word) of a row may reach into the row's padding
        constexpr int E = XFER / 2;
        const int64_t K8 = (pr.K + E - 1) & ~(E - 1), M8 = (pr.M + E - 1) & ~(E - 1), N8 = (pr.N + E - 1) & ~(E - 1);
        // A [row][k] operand's descriptor starts at the tile's first row and covers the tile's rows only, so
        // its range stays small however large the matrix is; a [k][row] operand's covers the k range.
        const int a_rows = min(BM, pr.M - m0), b_rows = min(BN, pr.N - n0);
        const int64_t a_elems = AKM ? ((int64_t)(a_rows - 1) * pr.lda + K8) : ((int64_t)(pr.K - 1) * pr.lda + M8);
        // a gathered B is described whole: any of the matrix's rows may be asked for
        const int64_t b_elems = pr.b_map ? ((int64_t)(pr.b_map_rows - 1) * pr.ldb + (BKM ? K8 : N8))
                                         : BKM ? ((int64_t)(b_rows - 1) * pr.ldb + K8) : ((int64_t)(pr.K - 1) * pr.ldb + N8);
        const uint16_t* a_base = (const uint16_t*)pr.A + (AKM ? (int64_t)m0 * pr.lda : 0);
        const uint16_t* b_base = (const uint16_t*)pr.B + ((BKM && !pr.b_map) ? (int64_t)n0 * pr.ldb : 0);
        ra = __builtin_amdgcn_make_buffer_rsrc((void*)a_base, 0, (int)(a_elems * 2), 0x00020000);
        rb = __builtin_amdgcn_make_buffer_rsrc((void*)b_base, 0, (int)(b_elems * 2), 0x00020000);
        constexpr int KS = 64 * SH::G;
        nk = (pr.K + KS - 1) / KS;
        const int k_first = 64 * group;
        // rows of a [row][k] operand beyond the tile (stage rows that only pad the tile included) lie beyond the
        // descriptor; of a [k][row] operand they are tested against the matrix
        pa.init(AKM, pr.lda, AKM ? 0 : m0, AKM ? min(BM, pr.M - m0) : min(pr.M, m0 + BM), pr.K, tid, k_first, KS, nk);
        if (pr.b_map && BKM)   // rows n0 .. of the product are rows b_map[n0 ..] of the matrix
            pb.init(true, pr.ldb, n0, min(pr.N, n0 + BN), pr.K, tid, k_first, KS, nk, pr.b_map, nullptr);
        else
            pb.init(BKM, pr.ldb, BKM ? 0 : n0, BKM ? min(BN, pr.N - n0) : min(pr.N, n0 + BN), pr.K, tid, k_first, KS, nk,
                    nullptr, ktab);
        fa.init(wm * SH::WTM, lane);
        fb.init(wn * SH::WTN, lane);
        smem = smem_ + group * SH::GROUP_BYTES;
        smem_addr = (uint32_t)(uintptr_t)FLOP_LDS_PTR(smem);
        const int last0 = (nk - 1) * KS + k_first;          // first k of this group's last step
        ktail = last0 + 64 > pr.K;
        kfix = pr.K & 7;
        const int straddle = pr.K & ~7;                     // first k of the chunk that straddles K
        kfix_chunk = (straddle >= last0 && straddle < last0 + 64) ? ((straddle - last0) >> 3) : -1;
    }

    // (a gathered B must have had its table entries of `step` fetched: pb.fetch_k)
    __device__ __forceinline__ void issue(int step) const
    {
        unsigned char* st = smem + (step % NB) * STAGE;
        const uint32_t tail_mask = (ktail && step == nk - 1) ? 0xFFFFFFFFu : 0u;
        pa.issue(ra, st, step, tail_mask, wave);
        pb.issue(rb, st + A_BYTES, step, tail_mask, wave);
    }

    // Transfers of stage t are complete once at most `later` younger stages are pending.
    __device__ __forceinline__ void wait_stage(int later) const
    {
        if (NB >= 6 && later >= 5) wait_vmcnt<(NB >= 6 ? 5 : 0) * LPS>();
        else if (NB >= 5 && later >= 4) wait_vmcnt<(NB >= 5 ? 4 : 0) * LPS>();
        else if (NB >= 4 && later >= 3) wait_vmcnt<(NB >= 4 ? 3 : 0) * LPS>();
        else if (NB >= 3 && later >= 2) wait_vmcnt<(NB >= 3 ? 2 : 0) * LPS>();
        else if (later >= 1) wait_vmcnt<LPS>();
        else wait_vmcnt<0>();
    }

    // K not a multiple of 8: in the last step the chunk that straddles K has brought
    // elements of the row padding into the k-major stage buffers; clear them (an
    // operand stored [k][row] needs nothing: its rows beyond K fail the range check).
    // Call with the stage landed and a barrier passed; the condition is the same for every
    // group of the block (they all reach the barrier inside), only the chunk's owner writes.
    __device__ __forceinline__ void fix_ktail(int step) const
    {
        if (kfix == 0 || step != nk - 1) return;
        unsigned char* st = smem + (step % NB) * STAGE;
        const int tid = threadIdx.x % (64 * SH::NWG);
        if (kfix_chunk >= 0) {
            if constexpr (AKM)
                for (int row = tid; row < BM; row += 64 * SH::NWG) {
                    uint16_t* c = (uint16_t*)(st + row * 128 + ((kfix_chunk ^ ((row >> 1) & 7)) << 4));
                    for (int e = kfix; e < 8; ++e) c[e] = 0;
                }
            if constexpr (BKM)
                for (int row = tid; row < BN; row += 64 * SH::NWG) {
                    uint16_t* c = (uint16_t*)(st + A_BYTES + row * 128 + ((kfix_chunk ^ ((row >> 1) & 7)) << 4));
                    for (int e = kfix; e < 8; ++e) c[e] = 0;
                }
        }
        __syncthreads();
    }

    __device__ __forceinline__ void read(int step, FragSet<TM, TN>& f) const
    {
        const uint32_t sa = smem_addr + (uint32_t)((step % NB) * STAGE);
        const uint32_t sb = sa + A_BYTES;
#define FLOP_KC_READ(KC)                                                                  \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) fa.template load<KC>(sa, i, f.a[KC][i]); \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) fb.template load<KC>(sb, j, f.b[KC][j]);
        FLOP_KC_READ(0)
        FLOP_KC_READ(1)
        FLOP_KC_READ(2)
        FLOP_KC_READ(3)
#undef FLOP_KC_READ
    }

    __device__ __forceinline__ void iterate(int s, FragSet<TM, TN>& cur, FragSet<TM, TN>& nxt,
                                            f32x16 (&acc)[TM][TN])
    {
        wait_fragset<TM, TN>(cur);
        pb.settle_k();
        if (s + 1 < nk) {
            // younger stages already issued: s+2 .. min(nk-1, s+NB-1)
            const int last = (nk - 1 < s + NB - 1) ? nk - 1 : s + NB - 1;
            wait_stage(last - (s + 1));
            __builtin_amdgcn_s_barrier();   // stage s+1 is complete in LDS; nobody still reads stage s
            if (s + NB < nk) {
                issue(s + NB);
                if (s + NB + 1 < nk) pb.fetch_k(s + NB + 1);
            }
            fix_ktail(s + 1);
            read(s + 1, nxt);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kc = 0; kc < 4; ++kc)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[kc][i].get(), cur.b[kc][j].get(),
                                                                       acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- steady-state iteration: LDS reads of step s+1 and the transfers of step s+NB are
    // issued one at a time in the shadow of the MFMAs of step s (an MFMA occupies the matrix
    // pipe for 8 passes but the issue port only briefly) ---------------------------------
    static constexpr int NMMA = 4 * TM * TN;        // MFMAs per step and wave
    static constexpr int NFRAG = 4 * (TM + TN);     // fragments per step and wave

    template <int F>
    __device__ __forceinline__ void read_frag(uint32_t sa, uint32_t sb, FragSet<TM, TN>& f) const
    {
        constexpr int KC = F / (TM + TN), IDX = F % (TM + TN);
        if constexpr (IDX < TM) fa.template load<KC>(sa, IDX, f.a[KC][IDX]);
        else fb.template load<KC>(sb, IDX - TM, f.b[KC][IDX - TM]);
    }

    template <int P>
    __device__ __forceinline__ void issue_transfer(unsigned char* st, int step, uint32_t tail_mask) const
    {
        if constexpr (P < PlanA::NV) pa.issue_one(P, ra, st, step, tail_mask, wave);
        else pb.issue_one(P - PlanA::NV, rb, st + A_BYTES, step, tail_mask, wave);
    }

    template <int M>
    __device__ __forceinline__ void slot(int s, uint32_t sa, uint32_t sb, unsigned char* st, uint32_t tail_mask,
                                         FragSet<TM, TN>& cur, FragSet<TM, TN>& nxt, f32x16 (&acc)[TM][TN]) const
    {
        constexpr int KC = M / (TM * TN), I = (M / TN) % TM, J = M % TN;
        acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[KC][I].get(), cur.b[KC][J].get(), acc[I][J], 0, 0, 0);
        // fragments M*NFRAG/NMMA .. (M+1)*NFRAG/NMMA - 1 of the next step
        constexpr int F0 = M * NFRAG / NMMA, F1 = (M + 1) * NFRAG / NMMA;
        if constexpr (F0 < F1) read_frag<F0>(sa, sb, nxt);
        if constexpr (F0 + 1 < F1) read_frag<F0 + 1>(sa, sb, nxt);
        if constexpr (F0 + 2 < F1) read_frag<F0 + 2>(sa, sb, nxt);
        static_assert(F1 - F0 <= 3, "too many fragments per MFMA slot");
        // the stage's transfers spread evenly over the slots
        constexpr int TPS = (LPS + NMMA - 1) / NMMA;
        static_assert(TPS <= 4, "too many transfers per MFMA slot");
        if constexpr (M * TPS < LPS) issue_transfer<(M * TPS < LPS ? M * TPS : 0)>(st, s + NB, tail_mask);
        if constexpr (TPS > 1 && M * TPS + 1 < LPS) issue_transfer<(M * TPS + 1 < LPS ? M * TPS + 1 : 0)>(st, s + NB, tail_mask);
        if constexpr (TPS > 2 && M * TPS + 2 < LPS) issue_transfer<(M * TPS + 2 < LPS ? M * TPS + 2 : 0)>(st, s + NB, tail_mask);
        if constexpr (TPS > 3 && M * TPS + 3 < LPS) issue_transfer<(M * TPS + 3 < LPS ? M * TPS + 3 : 0)>(st, s + NB, tail_mask);
        __builtin_amdgcn_sched_barrier(0);
    }

    template <int... Ms>
    __device__ __forceinline__ void slots(int s, uint32_t sa, uint32_t sb, unsigned char* st, uint32_t tail_mask,
                                          FragSet<TM, TN>& cur, FragSet<TM, TN>& nxt, f32x16 (&acc)[TM][TN],
                                          std::integer_sequence<int, Ms...>) const
    {
        (slot<Ms>(s, sa, sb, st, tail_mask, cur, nxt, acc), ...);
    }

    // valid while s + NB < nk - 1: every conditional of iterate() is taken and the
    // transfers issued are not the (possibly partial) last step
    __device__ __forceinline__ void iterate_steady(int s, FragSet<TM, TN>& cur, FragSet<TM, TN>& nxt,
                                                   f32x16 (&acc)[TM][TN])
    {
        wait_fragset<TM, TN>(cur);
        pb.settle_k();                  // table entries of step s+NB (gathered B), read during the last iteration
        wait_stage(NB - 2);             // stages s+2 .. s+NB-1 may still be in flight
        __builtin_amdgcn_s_barrier();   // stage s+1 is complete in LDS; nobody still reads stage s
        const uint32_t sa = smem_addr + (uint32_t)(((s + 1) % NB) * STAGE);
        unsigned char* st = smem + ((s + NB) % NB) * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        slots(s, sa, sa + A_BYTES, st, 0u, cur, nxt, acc, std::make_integer_sequence<int, NMMA>{});
        pb.fetch_k(s + NB + 1);         // in range: s + NB < nk - 1 here
    }

    __device__ __forceinline__ void run(f32x16 (&acc)[TM][TN])
    {
        FragSet<TM, TN> f0, f1;
#pragma unroll
        for (int s = 0; s < NB; ++s)
            if (s < nk) { pb.fetch_k(s); issue(s); }
        if (NB < nk) pb.fetch_k(NB);
        wait_stage((nk - 1 < NB - 1) ? nk - 1 : NB - 1);
        __builtin_amdgcn_s_barrier();
        fix_ktail(0);
        read(0, f0);
        int s = 0;
        for (; s + 2 + NB < nk; s += 2) {   // both iterations of the pair are steady
            iterate_steady(s, f0, f1, acc);
            iterate_steady(s + 1, f1, f0, acc);
        }
        for (; s < nk; s += 2) {
            iterate(s, f0, f1, acc);
            if (s + 1 < nk) iterate(s + 1, f1, f0, acc);
        }
    }
};

template <typename SH, bool AKM, bool BKM, int XFER>
__device__ __forceinline__ void dma_main_loop(const GemmProblem& pr, unsigned char* smem, int m0, int n0, int group,
                                              const uint16_t* ktab, f32x16 (&acc)[SH::TM][SH::TN])
{
    DmaLoop<SH, AKM, BKM, XFER> loop;
    loop.init(pr, smem, m0, n0, group, ktab);
    loop.run(acc);
}

// Measurement build (-DFLOP_PHASE_STAMPS, see flop_bench_phases_read): five wall-clock stamps per block.
#ifdef FLOP_PHASE_STAMPS
constexpr int kStampSlots = 16, kStampBlocks = 4096, kStampPhases = 5;
__device__ unsigned long long g_phase_stamps[kStampSlots * kStampBlocks * kStampPhases];
#define FLOP_STAMP(name) const unsigned long long name = wall_clock64()
#else
#define FLOP_STAMP(name)
#endif

template <typename SH, bool BKM, int XFER = 16>
__global__ __launch_bounds__(SH::THREADS) void gemm_bf16_dma_kernel(FLOP_HEAD_PARAMS, const GemmGroup grp)
{
    FLOP_STAMP(stamp_entry);
    constexpr int BM = SH::BM, BN = SH::BN, TM = SH::TM, TN = SH::TN, WTM = SH::WTM, WTN = SH::WTN;
    constexpr int THREADS = SH::THREADS, NWAVES = THREADS / 64;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    // (blocks of the first product do not look at the group before their main loop, see LaunchHead; the riders'
    // block indices lie beyond every product's)
    const bool head_block = (hflags & kHeadValid) != 0 && (int)(blockIdx.x >> 3) < hnext;
    if (!head_block && grp.rider_blocks > 0 && (int)blockIdx.x >= grp.tile_blocks) {   // block-uniform
        // the step-boundary blocks are written for kStreamThreads threads; surplus wavefronts leave
        if (THREADS > kStreamThreads && (int)threadIdx.x >= kStreamThreads) return;
        const int id = (int)blockIdx.x - grp.tile_blocks;
        step_boundary_block(grp.rider.fb, grp.rider.count, grp.rider.gj, id % grp.rider.bx, id / grp.rider.bx);
        return;
    }
    GemmProblem pr;
    int tile_m, tile_n;
    bool from_head;
    if (!(locate_tile<2, BM, BN>(FLOP_HEAD_ARGS, grp, pr, tile_m, tile_n, from_head))) return;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int group = __builtin_amdgcn_readfirstlane(wave / SH::NWG);
    const int wig = wave % SH::NWG;                       // wavefront inside its group
    const int wm = wig / SH::WN, wn = wig % SH::WN;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // B gathered along k: the matrix rows of its k rows go to a table behind the block's other LDS (block-uniform
    // condition; the host has checked K <= kKtabMaxK and fewer than 65535 rows)
    const uint16_t* ktab = nullptr;
    if constexpr (!BKM && XFER == 16) {
        if (pr.b_map) {
            uint16_t* tab = (uint16_t*)(smem + gemm_dma_lds_bytes<SH>());
            constexpr int KS = 64 * SH::G;
            const int entries = (pr.K + KS - 1) / KS * KS;
            for (int k = tid; k < entries; k += THREADS)
                tab[k] = (uint16_t)(k < pr.K ? (uint32_t)pr.b_map[k] : kKtabNone);
            __syncthreads();
            ktab = tab;
        }
    }
    // the remaining fields of a head block's product: requested here, first needed after the main loop, so the
    // trip to the kernel-argument segment passes while the first stages are on their way
    FLOP_STAMP(stamp_setup);
    constexpr bool kEarlyTail = SH::THREADS <= 384 && XFER == 16;   // (the other kernels have no registers to spare)
    if (kEarlyTail && from_head) finish_problem(pr, grp.p[0]);
    if (pr.a_kmajor) dma_main_loop<SH, true, BKM, XFER>(pr, smem, m0, n0, group, ktab, acc);
    else dma_main_loop<SH, false, BKM, XFER>(pr, smem, m0, n0, group, ktab, acc);
    __syncthreads();
    FLOP_STAMP(stamp_loop);
    if (!kEarlyTail && from_head) finish_problem(pr, grp.p[0]);

    // ---- the groups' partial sums are added in group order (fixed, so the result is deterministic): groups
    // 1 .. G-1 leave theirs in LDS, lane-interleaved, group 0 adds them up and goes on alone
    if constexpr (SH::G > 1) {
        float* part = (float*)smem;
        constexpr int PER_WAVE = TM * TN * 16 * 64;      // floats a wavefront holds
        if (group > 0) {
            float* mine = part + ((group - 1) * SH::NWG + wig) * PER_WAVE + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mine[((i * TN + j) * 16 + v) * 64] = acc[i][j][v];
        }
        __syncthreads();
        if (group == 0) {
#pragma unroll
            for (int gg = 1; gg < SH::G; ++gg) {
                const float* theirs = part + ((gg - 1) * SH::NWG + wig) * PER_WAVE + lane;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][j][v] += theirs[((i * TN + j) * 16 + v) * 64];
            }
        }
        __syncthreads();
    }

    // ---- k-split launch: this block's float32 partial sums, unscaled; a later kernel adds the slices
    if (pr.ksplit > 1) {
        if (group == 0) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * WTN + j * 32 + l32;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = m0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                        if (row < pr.M && col < pr.N) pr.split_out[(int64_t)row * pr.N + col] = acc[i][j][v];
                    }
            }
        }
        return;
    }

    // ---- epilogue ------------------------------------------------------------------
    // Output tile: gate scale, one rounding to bfloat16, staged in LDS as [row][col]
    // (rows padded by 16 bytes), then written with 16-byte row-contiguous stores.
    // The first ACTIVE threads each own chunk column cc of the rows row_t, row_t + RSTEP, ...; with
    // pr.dot they also add up C .* dot over those rows for their 8 columns.
    constexpr int PITCH = BN * 2 + 16;
    constexpr int CPR = BN / 8;                    // 16-byte chunks per tile row
    constexpr int RSTEP_MAX = THREADS / CPR;       // rows that the block's threads cover in one pass
    constexpr int RSTEP = (BM % RSTEP_MAX == 0) ? RSTEP_MAX : (BM % (RSTEP_MAX / 2) == 0 ? RSTEP_MAX / 2 : RSTEP_MAX / 4);
    constexpr int ACTIVE = RSTEP * CPR;            // threads that store (all of them unless BN / 8 does not divide the block)
    constexpr int NCH = BM / RSTEP;                // chunks per storing thread
    static_assert(RSTEP >= 1 && BM % RSTEP == 0 && ACTIVE <= THREADS, "chunk ownership");
    const bool storing = tid < ACTIVE;
    const int cc = tid % CPR, row_t = tid / CPR;
    const int ccol = n0 + cc * 8;
    const bool dot = pr.dot_partial != nullptr;
    const bool dot_vec = (((uintptr_t)pr.dot & 15u) == 0) && (pr.lddot % 8 == 0);
    u32x4 gq[NCH];
    if (dot && storing) {
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int row = m0 + row_t + q * RSTEP;
            gq[q] = u32x4{0u, 0u, 0u, 0u};
            if (row < pr.M && ccol < pr.N) {
                const uint16_t* src = (const uint16_t*)pr.dot + (int64_t)row * pr.lddot + ccol;
                if (dot_vec) {
                    gq[q] = *(const u32x4*)src;
                } else {   // rows only 4-byte aligned (N even): whole words up to the end of the row, no further -
                           // a dense last row ends the matrix
                    const uint32_t* w = (const uint32_t*)src;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ccol + 2 * e < pr.N) gq[q][e] = w[e];
                }
            }
        }
    }
    if (group == 0) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col_l = wn * WTN + j * 32 + l32;
            const int col = n0 + col_l;
            float scale = 1.0f;
            if (col < pr.N) {
                if (pr.gate_alpha) {   // the gate itself, bit for bit what the gate kernels write for the same inputs
                    float dd;
                    gate_one(pr.gate_alpha[col], pr.gate_u[col], 1.0f / pr.gate_beta, pr.gate_l, pr.gate_r, 0, scale, dd);
                } else if (pr.col_scale) {
                    scale = pr.col_scale[col];
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row_l = wm * WTM + i * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                    *(uint16_t*)(smem + row_l * PITCH + col_l * 2) = (uint16_t)f32_to_bf16_bits(acc[i][j][v] * scale);
                }
        }
    }
    __syncthreads();
    FLOP_STAMP(stamp_staged);
    const bool c_vec = (((uintptr_t)pr.C & 15u) == 0) && (pr.ldc % 8 == 0);
    const bool c_word = (((uintptr_t)pr.C & 3u) == 0) && (pr.ldc % 2 == 0);   // rows 4-byte aligned
    float ds[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ds[e] = 0.0f;
    if (storing) {
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int row_l = row_t + q * RSTEP;
            const int row = m0 + row_l;
            if (row >= pr.M || ccol >= pr.N) continue;
            const u32x4 v = *(const u32x4*)(smem + row_l * PITCH + cc * 16);
            const int64_t orow = pr.c_rowmap ? pr.c_rowmap[row] : row;
            uint16_t* dst = (uint16_t*)pr.C + orow * pr.ldc + ccol;
            if (c_vec && ccol + 8 <= pr.N) {
                __builtin_nontemporal_store(v, (u32x4*)dst);
            } else if (c_word && ccol + 8 <= pr.N) {
                ((uint32_t*)dst)[0] = v[0]; ((uint32_t*)dst)[1] = v[1];
                ((uint32_t*)dst)[2] = v[2]; ((uint32_t*)dst)[3] = v[3];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (ccol + e < pr.N) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
            }
            if (dot) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t vw = v[e >> 1], gw = gq[q][e >> 1];
                    const float cv = __builtin_bit_cast(float, (e & 1) ? (vw & 0xFFFF0000u) : (vw << 16));
                    const float gv = __builtin_bit_cast(float, (e & 1) ? (gw & 0xFFFF0000u) : (gw << 16));
                    if (ccol + e < pr.N) ds[e] = fmaf(cv, gv, ds[e]);
                }
            }
        }
    }
    if (dot) {
        // Column sums of the tile: every thread leaves its eight in LDS (threads that stored nothing leave
        // zeros), then thread n adds column n over the RSTEP row lanes in a fixed order.
        float* red = (float*)(smem + ((BM * PITCH + 15) & ~15));
        if (storing) {
#pragma unroll
            for (int e = 0; e < 8; ++e) red[row_t * BN + cc * 8 + e] = ds[e];
        }
        __syncthreads();
        if (tid < BN && n0 + tid < pr.N) {
            float tot = 0.0f;
#pragma unroll 8
            for (int q = 0; q < RSTEP; ++q) tot += red[q * BN + tid];
            pr.dot_partial[(int64_t)tile_m * pr.dot_ld + n0 + tid] = tot;
        }
    }
#ifdef FLOP_PHASE_STAMPS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the block's stores have been acknowledged
    if (threadIdx.x == 0 && grp.stamp_slot >= 0 && grp.stamp_slot < kStampSlots && (int)blockIdx.x < kStampBlocks) {
        unsigned long long* o = g_phase_stamps + ((size_t)grp.stamp_slot * kStampBlocks + blockIdx.x) * kStampPhases;
        o[0] = stamp_entry; o[1] = stamp_setup; o[2] = stamp_loop; o[3] = stamp_staged; o[4] = wall_clock64();
    }
#endif
}

template <typename SH>
constexpr size_t gemm_dma_lds_bytes()
{
    constexpr int THREADS = SH::THREADS, CPR = SH::BN / 8, RSTEP_MAX = THREADS / CPR;
    const size_t stages = (size_t)SH::G * SH::GROUP_BYTES;
    const size_t partials = (size_t)(SH::G - 1) * SH::BM * SH::BN * sizeof(float);
    const size_t out_tile = (size_t)SH::BM * (SH::BN * 2 + 16) + 16 + (size_t)RSTEP_MAX * SH::BN * sizeof(float);   // + column-sum lanes
    size_t m = stages > out_tile ? stages : out_tile;
    return m > partials ? m : partials;
}

}  // namespace flop
