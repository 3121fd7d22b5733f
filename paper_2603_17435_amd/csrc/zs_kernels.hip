// HIP kernels and device entry points of libzipserv_hip.so (gfx950 only).
//   zs_decompress : TCA-TBE blob -> row-major BF16 (standalone kernel, Section 4.4)
//   zs_gemm       : C = A * decode(W)^T, decode fused into the MFMA loop (ZipGEMM, Section 4.3)
//
// Both kernels are built from independent waves.  A wave streams BlockTiles: the compressed
// bytes of the next DEPTH - 1 tiles are in flight from HBM straight into LDS
// (global_load_lds_dwordx4, the "tile loading" stage of Section 4.3.1) while the current tile
// is decoded from LDS into registers (Algorithm 2) and, in ZipGEMM, multiplied on the matrix
// cores.  No barrier is needed inside the stream: a wave only reads what it staged itself.
#include <hip/hip_runtime.h>

#include <cstring>
#include <type_traits>

#include "zipserv.h"
#include "zs_device.h"

using namespace zs;

namespace {

constexpr int kNumCus = 256;
constexpr uint32_t kMaxLds = 160 * 1024;

// ---- slot = LDS image of one BlockTile -------------------------------------------------
//   [0, 1536)            bit-planes
//   [1536, 5632)         H segment (at most 4096 bytes)
//   [5632, +LW)          first LW bytes of the L segment (LW = 512, 1024 or 4096)
//   64 bytes of slack    for the aligned over-read of the byte gathers
template <int LW>
struct Slot {
    static constexpr uint32_t kPlanes = 0, kH = ZS_BT_BITMAP_BYTES, kL = kH + 4096;
    static constexpr uint32_t kBytes = kL + LW + 64;
    static constexpr int kLChunks = (LW + 1023) / 1024;
    static constexpr int kLoads = 2 + 4 + kLChunks; // LDS-direct instructions per BlockTile
};

struct Segments {
    const uint8_t *h, *l;
    uint32_t h_bytes, l_bytes;
    uint32_t h_room, l_room; // 16-byte units from the segment's start to the end of its section
};

// The two offset pairs that bracket BlockTile bt.  The offset array is read-only for the whole
// launch: reading it through the constant address space lets a wave-uniform index use scalar
// loads, which do not share the vector-memory counter with the LDS-direct loads.
struct OffsetPairs {
    u32x2 o0, o1;
};
__device__ __forceinline__ OffsetPairs offset_pairs(const BlobView &bv, uint32_t bt)
{
    typedef const u32x2 __attribute__((address_space(4))) *ConstPairs;
    const ConstPairs off = (ConstPairs)(uintptr_t)bv.offsets;
    return OffsetPairs{off[bt], off[bt + 1]};
}

// Start and size of a BlockTile's H and L segments, clamped so that no read can leave the
// blob sections or a slot whatever the offset array holds.
__device__ __forceinline__ Segments segments_from(const BlobView &bv, const OffsetPairs &o)
{
    const uint32_t h0 = min(o.o0.x, bv.h_units), l0 = min(o.o0.y, bv.l_units);
    const uint32_t h1 = min(max(o.o1.x, h0), bv.h_units), l1 = min(max(o.o1.y, l0), bv.l_units);
    Segments s;
    s.h = bv.H + (size_t)h0 * 16;
    s.l = bv.L + (size_t)l0 * 16;
    s.h_bytes = min(h1 - h0, (uint32_t)(ZS_BT_ELEMS / 16)) * 16;
    s.l_bytes = min(l1 - l0, (uint32_t)(2 * ZS_BT_ELEMS / 16)) * 16;
    s.h_room = bv.h_units - h0;
    s.l_room = bv.l_units - l0;
    return s;
}
__device__ __forceinline__ Segments segments_of(const BlobView &bv, uint32_t bt)
{
    return segments_from(bv, offset_pairs(bv, bt));
}

// Issues the Slot::kLoads LDS-direct loads of BlockTile bt (exactly that many instructions,
// also when !valid: then only lane 0 runs, on a dummy address).
template <int LW>
__device__ __forceinline__ void issue_block_tile(const BlobView &bv, uint32_t bt, bool valid, uint32_t slot_at,
                                                 uint32_t lane)
{
    using S = Slot<LW>;
    Segments sg = {bv.H, bv.L, 0u, 0u, 0u, 0u};
    if (valid) sg = segments_of(bv, bt);
    const uint8_t *planes = bv.bitmaps + (size_t)(valid ? bt : 0u) * ZS_BT_BITMAP_BYTES;
    dma_segment<2>(planes, valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane * 16, bv.bitmaps);
    dma_segment<4>(sg.h, sg.h_bytes, slot_at + S::kH, lane * 16, bv.bitmaps);
    dma_segment<S::kLChunks>(sg.l, min(sg.l_bytes, (uint32_t)LW), slot_at + S::kL, lane * 16, bv.bitmaps);
}

__device__ __forceinline__ uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

// LDS address of the dynamic shared array: it follows the kernel's static LDS (a link-time
// constant; these kernels have none).  Taking the address through a pointer cast instead
// leaves a null-pointer select at every use.
__device__ __forceinline__ uint32_t dynamic_lds_base() { return __builtin_amdgcn_groupstaticsize(); }

// --------------------------------------------------------------------------------------
// Standalone decompression: waves take BlockTiles round-robin; 16 bytes (8 weights) per lane
// and TensorCoreTile are stored row-major.
// --------------------------------------------------------------------------------------
template <int LW, int DEPTH, int WAVES, bool BASE_M1>
__global__ __launch_bounds__(64 * WAVES) void decompress_kernel(BlobView bv, uint16_t *out, int64_t ldw)
{
    using S = Slot<LW>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables(smem, bv.base_exp);
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = dynamic_lds_base();
    const uint32_t ring = tab + kTableBytes + wave * (DEPTH * S::kBytes);
    const uint32_t n_bt = (uint32_t)bv.strips * (uint32_t)bv.k_blocks;
    const uint32_t first = blockIdx.x * WAVES + wave, stride = gridDim.x * WAVES;
    const uint32_t row_in_tt = ((lane >> 3) & 1u) * 8u + (lane & 7u); // FragTiles run N-fastest
    const uint32_t col_in_tt = (lane >> 4) * 8u;

#pragma unroll
    for (int j = 0; j < DEPTH - 1; ++j) {
        const uint32_t bt = first + j * stride;
        issue_block_tile<LW>(bv, bt, bt < n_bt, ring + j * S::kBytes, lane);
    }
    uint32_t cur = 0, nxt = DEPTH - 1; // ring positions of the tile being decoded / being issued
    for (uint32_t bt = first; bt < n_bt; bt += stride) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // every LDS read of the slot about to be refilled is done
        const uint32_t ahead = bt + (DEPTH - 1) * stride;
        issue_block_tile<LW>(bv, ahead, ahead < n_bt, ring + nxt * S::kBytes, lane);
        wait_dma<(DEPTH - 1) * S::kLoads>();

        const uint32_t slot = ring + cur * S::kBytes;
        const Segments sg = segments_of(bv, bt);
        BlockIndex bi;
        index_read_planes(slot + S::kPlanes, lane, bi);
        index_block_tile(slot + S::kH, slot + S::kL, lane, bi);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(sg.l), sg.l_bytes > (uint32_t)LW};
        const uint32_t strip = bt / (uint32_t)bv.k_blocks, kb = bt % (uint32_t)bv.k_blocks;
        uint16_t *dst = out + ((int64_t)strip * 64 + row_in_tt) * ldw + (int64_t)kb * 64 + col_in_tt;
        auto run = [&](auto careful) {
            decode_block_tile<BASE_M1, decltype(careful)::value, true>(tab, bi, fs, [&](int tt, const u32x4 &w) {
                __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(dst + (int64_t)((tt & 3) * 16) * ldw + (tt >> 2) * 32));
            });
        };
        // rows with three or more fallbacks (or an over-long L segment) take the careful variant
        if (fs.from_global || __builtin_amdgcn_ballot_w64(bi.min_cnt < 6) != 0)
            run(std::true_type{});
        else
            run(std::false_type{});
        cur = cur + 1 == DEPTH ? 0 : cur + 1;
        nxt = nxt + 1 == DEPTH ? 0 : nxt + 1;
    }
    wait_dma<0>();
}

// --------------------------------------------------------------------------------------
// ZipGEMM, skinny-M regime.  W is the MFMA A operand (rows = output features), the
// activations are the B operand (columns = tokens, 16 per MFMA, MT MFMAs per weight tile).
//
// Work split (a refinement of the split-K tiling of Section 4.3.1): the BlockTiles of the
// matrix, in storage order (K-fastest inside 64-row strips), form one sequence that is cut
// into gridDim.x equal contiguous ranges, one per workgroup, wherever the cuts fall.  The
// part of a strip inside a range is a task (tasks are numbered locally, j = 0, 1, ..., in the
// order they are processed: the range's last strip first, then from its beginning).
//
// Inside a workgroup WAVES streaming waves take BlockTiles from the range one at a time off
// a shared counter (so a wave that shares its SIMD with fewer others simply takes more), each
// staging its next tile with LDS-direct loads while it decodes and multiplies the current one.
// A wave keeps the 64 x (16 MT) FP32 partial sums of one task in registers; when its next
// tile belongs to another task it adds them, under a lock, into that task's accumulation
// tile in LDS (two tiles, by parity of j) and reports how many BlockTiles they covered.  One
// more wave, the writer, waits until a task's count is complete, takes the tile out of LDS,
// hands the LDS tile back and stores it to C when the task is a whole strip.  The tile of a
// strip shared with other workgroups goes to global scratch instead, and the last workgroup
// to contribute adds the tiles up and stores the strip (without scratch memory: FP32 atomics
// onto a C cleared beforehand).  Streaming waves never meet at a barrier.
//
// The activations of a 64-wide K slab (L2-resident) are loaded straight from A into registers,
// in B-operand lane order, one tile ahead: right after the LDS-direct loads of the tile they
// belong to.
// --------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) uint32_t *LdsU32;
typedef __attribute__((address_space(3))) f32x4 *LdsF32x4;

__device__ __forceinline__ uint32_t lds_poll(uint32_t at)
{
    return __hip_atomic_load((LdsU32)at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// The six LDS-direct loads of the bit-planes and H of a tile whose H segment has 4096 readable
// bytes after its start (whatever its own length: what lies beyond belongs to the next tiles
// and is ignored).  No per-chunk address or lane-mask arithmetic is needed then: two base
// registers, instruction offsets, and a lane mask for the last H chunk only (k3, at least
// lane 0).  Nothing is waited for.  All operands except lane16 (= 16 * lane) are
// wave-uniform; all 64 lanes must be active.
__device__ __forceinline__ void stage_fast6(uint32_t lane16, uint32_t slot_at, const uint8_t *planes, const uint8_t *h,
                                            uint64_t k3)
{
    static_assert(ZS_BT_BITMAP_BYTES == 1536, "the LDS offsets below assume 1536 bytes of bit-planes");
    asm volatile("s_mov_b32 m0, %[slot]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[l16], %[bp]\n\t"
                 "s_mov_b64 exec, %[kp]\n\tglobal_load_lds_dwordx4 %[l16], %[bp] offset:1024\n\t"
                 "s_mov_b64 exec, -1\n\ts_add_u32 m0, %[slot], 1536\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %[l16], %[bh]\n\tglobal_load_lds_dwordx4 %[l16], %[bh] offset:1024\n\t"
                 "global_load_lds_dwordx4 %[l16], %[bh] offset:2048\n\ts_mov_b64 exec, %[k3]\n\t"
                 "global_load_lds_dwordx4 %[l16], %[bh] offset:3072\n\ts_mov_b64 exec, -1"
                 :
                 : [l16] "v"(lane16), [slot] "s"(slot_at), [bp] "s"(planes), [bh] "s"(h), [k3] "s"(k3),
                   [kp] "s"(0xFFFFFFFFull)
                 : "memory", "scc");
}

#ifdef ZS_DBG_TIMING
// debug builds only: accumulate cycle-counter deltas between marks into zs_t[]
#define ZS_T(i) { lds_fence(); uint64_t now = __builtin_readcyclecounter(); if (i > 0) zs_t[i] += now - zs_last; else zs_t[5] += 1; zs_last = now; }
#else
#define ZS_T(i)
#endif

// Control words in LDS (byte offsets from the control block).
enum : uint32_t { kCtlNext = 0, kCtlWritten = 4, kCtlLock = 8, kCtlDone = 16, kCtlBytes = 64 };

// Global scratch for strips that several workgroups contribute to.  A shared strip is counted
// in count[b], b = the first workgroup that contributes to it (unique: a range that holds the
// starts of two strips holds the first of them whole); the words are zero between launches
// (the workgroup that finishes a strip resets its counter).  tiles holds two partial tiles
// per workgroup (its first and its last task), each 64 rows x 16 MT tokens of FP32.
// count == nullptr selects the fallback: FP32 atomics onto a C cleared beforehand.
struct SharedSums {
    uint32_t *count;
    float *tiles;
};

// The BlockTile sequence [0, total) is cut into `parts` ranges; range b starts at
// floor(total * b / parts).
__device__ __forceinline__ uint32_t range_begin(uint32_t b, uint32_t total, uint32_t parts)
{
    return (uint32_t)((uint64_t)total * b / parts);
}
// The range that BlockTile g lies in.
__device__ __forceinline__ uint32_t range_of(uint32_t g, uint32_t total, uint32_t parts)
{
    uint32_t b = (uint32_t)((uint64_t)g * parts / total);
    while (b + 1 < parts && range_begin(b + 1, total, parts) <= g) ++b;
    while (range_begin(b, total, parts) > g) --b;
    return b;
}

template <int MT, int LW, int WAVES, bool BASE_M1>
__global__ __launch_bounds__(64 * (WAVES + 1)) void gemm_stream_kernel(BlobView bv, const uint16_t *A, int64_t lda,
                                                                  float *C, int64_t ldc, int M, SharedSums ws,
                                                                  uint64_t *dbg)
{
    (void)dbg;
    constexpr int DEPTH = 2; // ring positions per wave: one tile decoded, one in flight
    using S = Slot<LW>;
    // LDS after the tables: two accumulation tiles (16 MT tokens x 64 rows, FP32, in units of
    // float4 = 4 consecutive rows; unit (m, c) lives at m * 16 + (c ^ (m & 15)) so that the 16
    // tokens of one MFMA result hit 16 different bank groups), the control words, the rings.
    constexpr uint32_t kUnits = 16 * MT * 16, kTileBytes = 16 * kUnits;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
#ifdef ZS_DBG_TIMING
    const uint64_t zs_entry = __builtin_readcyclecounter();
#endif
    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = dynamic_lds_base();
    const uint32_t red = tab + kTableBytes, ctl = red + 2 * kTileBytes;
    const uint32_t ring = ctl + kCtlBytes + wave * (DEPTH * S::kBytes);
    const uint32_t m_lane = lane & 15u, kgrp = lane >> 4;
    // B operand of the 16x16x32 MFMA: lane l holds token l % 16 and the 8 consecutive k that
    // start at 8 * (l / 16).  Tokens >= M read token 0 instead (their columns are never stored).
    uint32_t rowoff[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        const uint32_t m = j * 16 + m_lane;
        rowoff[j] = ((int)m < M ? m : 0u) * (uint32_t)lda * 2u + kgrp * 16u;
    }

    // this workgroup's range [g0, g1) of the BlockTile sequence and its tasks
    const uint32_t k_blocks = (uint32_t)bv.k_blocks, total = (uint32_t)bv.strips * k_blocks;
    const uint32_t g0 = range_begin(blockIdx.x, total, gridDim.x), g1 = range_begin(blockIdx.x + 1, total, gridDim.x);
    const uint32_t strip0 = g0 / k_blocks;
    if (g0 >= g1) return;
    // Processing order: a range that touches several strips starts with its last one and then
    // runs from its beginning.  The (possibly shared) strips at both ends of the range are
    // then finished early, and what shared strips cost on top (parking the partial tile in
    // global memory, counting in, summing up) overlaps with the remaining work instead of
    // standing at the end of the kernel.  Tasks are numbered in processing order; the counter
    // that hands out BlockTiles counts positions c = 0 .. g1 - g0 - 1 in that order.
    const uint32_t strip_last = (g1 - 1) / k_blocks, n_tasks = strip_last - strip0 + 1;
    const uint32_t rot = n_tasks > 1 ? g1 - strip_last * k_blocks : 0u; // BlockTiles taken before g0
    auto task_strip = [&](uint32_t j) { return rot ? (j ? strip0 + j - 1 : strip_last) : strip0 + j; };

    // ---- issuing side: takes the next BlockTile off the shared counter and looks up its segments
    uint32_t it_j = rot ? 1u : 0u, it_base = strip0 * k_blocks; // task and first BlockTile of the strip the counter is in
    bool p_valid = false;                           // the next BlockTile to issue ...
    uint32_t p_g = 0, p_j = 0, p_kb = 0;
    Segments p_sg = {bv.H, bv.L, 0u, 0u, 0u, 0u}; // ... and its segments
    // Taking the next BlockTile is spread over three points of a step so that neither the LDS
    // atomic nor the scalar loads are waited for where they are issued.
    uint32_t g_taken = 0; // (per lane) what the counter returned
    OffsetPairs p_off = {u32x2{0u, 0u}, u32x2{0u, 0u}};
    auto take_begin = [&]() {
        g_taken = 0;
        if (lane == 0)
            g_taken = __hip_atomic_fetch_add((LdsU32)(ctl + kCtlNext), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto take_lookup = [&]() {
        const uint32_t c = uniform(g_taken);
        p_valid = c < g1 - g0;
        if (p_valid) {
            if (c < rot) { // the range's last strip, task 0
                p_g = strip_last * k_blocks + c, p_j = 0, p_kb = c;
            } else {
                const uint32_t g = g0 + (c - rot);
                while (g - it_base >= k_blocks) it_base += k_blocks, ++it_j;
                p_g = g, p_j = it_j, p_kb = g - it_base;
            }
            p_off = offset_pairs(bv, p_g);
        }
    };
    auto take_finish = [&]() {
        p_sg = Segments{bv.H, bv.L, 0u, 0u, 0u, 0u};
        if (p_valid) p_sg = segments_from(bv, p_off);
    };
    // what the decoding side needs to know about a staged tile, per ring position (wave-uniform)
    bool s_valid[DEPTH];
    uint32_t s_j[DEPTH], s_kb[DEPTH];
    const uint8_t *s_l[DEPTH];
    bool s_big[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) s_valid[d] = false, s_j[d] = 0, s_kb[d] = 0, s_l[d] = bv.L, s_big[d] = false;
    auto note = [&](int d) {
        s_valid[d] = p_valid, s_j[d] = p_j, s_kb[d] = p_kb, s_l[d] = p_sg.l, s_big[d] = p_sg.l_bytes > (uint32_t)LW;
    };

    // The first BlockTile of every streaming wave is assigned statically (position = wave) and
    // staged before anything else: its loads are in flight while the tables are built.
    if (wave < WAVES) {
        g_taken = wave;
        take_lookup();
        take_finish();
        const uint32_t slot_at = ring;
        const uint8_t *planes = bv.bitmaps + (size_t)(p_valid ? p_g : 0u) * ZS_BT_BITMAP_BYTES;
        dma_segment<2>(planes, p_valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane * 16, bv.bitmaps);
        dma_segment<4>(p_sg.h, p_sg.h_bytes, slot_at + S::kH, lane * 16, bv.bitmaps);
        dma_segment<S::kLChunks>(p_sg.l, min(p_sg.l_bytes, (uint32_t)LW), slot_at + S::kL, lane * 16, bv.bitmaps);
        note(0);
    }
    build_tables(smem, bv.base_exp);
    for (uint32_t i = threadIdx.x; i < (2 * kTileBytes + kCtlBytes) / 4; i += blockDim.x)
        *((LdsU32)(red + 4 * i)) = i == (2 * kTileBytes + kCtlNext) / 4 ? (uint32_t)WAVES : 0u;
    __syncthreads();

    // ---- the last wave of the workgroup only writes results.  Stores count in the same
    //      vector-memory counter as the LDS-direct loads, and a store is acknowledged late while
    //      HBM is saturated with reads; a streaming wave that stored would stall its own pipeline.
    if (wave == WAVES) {
        for (uint32_t j = 0; j < n_tasks; ++j) {
            const uint32_t strip = task_strip(j), par = j & 1u, tile = red + par * kTileBytes;
            const uint32_t lo = max(g0, strip * k_blocks), hi = min(g1, (strip + 1) * k_blocks);
            while (uniform(lds_poll(ctl + kCtlDone + 4 * par)) != hi - lo) __builtin_amdgcn_s_sleep(4);
            lds_fence();
            f32x4 v[kUnits / 64];
#pragma unroll
            for (uint32_t q = 0; q < kUnits / 64; ++q) {
                const uint32_t u = q * 64 + lane, m = u >> 4, c = u & 15u;
                const LdsF32x4 at = (LdsF32x4)(tile + 16 * (m * 16 + (c ^ (m & 15u))));
                v[q] = *at;
                *at = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            lds_fence(); // the tile is read and cleared: hand it back
            if (lane == 0) {
                __hip_atomic_store((LdsU32)(ctl + kCtlDone + 4 * par), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                lds_fence();
                __hip_atomic_store((LdsU32)(ctl + kCtlWritten), j + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            const bool whole = hi - lo == k_blocks;
            if (!whole && ws.count) {
                // A strip shared with other workgroups, summed without atomics on C: every
                // contributor parks its partial tile in global scratch and counts itself in;
                // whoever counts last adds the tiles up in workgroup order and stores the strip.  Scratch and counter are
                // accessed with agent-scope atomics, which are coherent between the L2s of
                // the chip's dies without cache-wide write-backs or invalidations.
                float *mine = ws.tiles + (size_t)(2 * blockIdx.x + (strip == strip0 ? 0u : 1u)) * (kUnits * 4);
#pragma unroll
                for (uint32_t q = 0; q < kUnits / 64; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        __hip_atomic_store(mine + (q * 64 + lane) * 4 + e, v[q][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // the tile has arrived before it is counted
                const uint32_t b_lo = range_of(strip * k_blocks, total, gridDim.x);
                const uint32_t b_hi = range_of((strip + 1) * k_blocks - 1, total, gridDim.x);
                uint32_t old = 0;
                if (lane == 0) old = __hip_atomic_fetch_add(ws.count + b_lo, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (uniform(old) != b_hi - b_lo) continue; // somebody else will finish the strip
                f32x4 sum[kUnits / 64];
#pragma unroll
                for (uint32_t q = 0; q < kUnits / 64; ++q) sum[q] = f32x4{0.f, 0.f, 0.f, 0.f};
                for (uint32_t b = b_lo; b <= b_hi; ++b) {
                    if (b == blockIdx.x) {
#pragma unroll
                        for (uint32_t q = 0; q < kUnits / 64; ++q) sum[q] += v[q];
                        continue;
                    }
                    // slot 0 of a workgroup holds the strip its range starts in, slot 1 the one it ends in
                    const uint32_t first = range_begin(b, total, gridDim.x) >= strip * k_blocks ? 0u : 1u;
                    const float *part = ws.tiles + (size_t)(2 * b + first) * (kUnits * 4);
#pragma unroll
                    for (uint32_t q = 0; q < kUnits / 64; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            sum[q][e] += __hip_atomic_load(part + (q * 64 + lane) * 4 + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (lane == 0) __hip_atomic_store(ws.count + b_lo, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (uint32_t q = 0; q < kUnits / 64; ++q) v[q] = sum[q];
            }
#pragma unroll
            for (uint32_t q = 0; q < kUnits / 64; ++q) {
                const uint32_t u = q * 64 + lane, m = u >> 4, c = u & 15u;
                if ((int)m < M) {
                    float *dst = C + (int64_t)m * ldc + (int64_t)strip * 64 + 4 * c;
                    if (whole || ws.count) {
                        *reinterpret_cast<f32x4 *>(dst) = v[q];
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dst + e, v[q][e]);
                    }
                }
            }
        }
        return;
    }

    f32x4 acc[4][MT];
    auto clear_acc = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
#ifdef ZS_DBG_TIMING
    uint64_t zs_t[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, zs_last = 0;
    zs_t[7] = __builtin_readcyclecounter();
#endif
    // Adds the partial sums of n BlockTiles of task j into the task's LDS tile.  D layout of the
    // 16x16 MFMA: a lane holds token lane % 16 and rows 4 * (lane / 16) .. + 3 of the 16-row
    // block, i.e. one float4 unit.
    auto flush = [&](uint32_t j, uint32_t n) {
#ifdef ZS_DBG_TIMING
        const uint64_t zs_r0 = __builtin_readcyclecounter();
#endif
        const uint32_t par = j & 1u, tile = red + par * kTileBytes;
        // the tile may still hold task j - 2: wait until the writer has handed it back
        while ((int32_t)uniform(lds_poll(ctl + kCtlWritten)) + 1 < (int32_t)j) __builtin_amdgcn_s_sleep(2);
        for (;;) {
            uint32_t old = 1;
            if (lane == 0) {
                uint32_t expect = 0;
                __hip_atomic_compare_exchange_strong((LdsU32)(ctl + kCtlLock + 4 * par), &expect, 1u, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                old = expect;
            }
            if (uniform(old) == 0) break;
            __builtin_amdgcn_s_sleep(1);
        }
        lds_fence();
#pragma unroll
        for (int jj = 0; jj < MT; ++jj)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t m = jj * 16 + m_lane, c = i * 4 + kgrp;
                const LdsF32x4 at = (LdsF32x4)(tile + 16 * (m * 16 + (c ^ (m & 15u))));
                *at = *at + acc[i][jj];
            }
        lds_fence(); // sums written before the lock opens and the count rises
        if (lane == 0) {
            __hip_atomic_store((LdsU32)(ctl + kCtlLock + 4 * par), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_add((LdsU32)(ctl + kCtlDone + 4 * par), n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
#ifdef ZS_DBG_TIMING
        zs_t[10] += __builtin_readcyclecounter() - zs_r0;
        zs_t[11] += 1;
#endif
    };

    take_begin();
    take_lookup();
#ifdef ZS_DBG_TIMING
    zs_t[8] = __builtin_readcyclecounter();
#endif
    clear_acc();
    uint32_t acc_j = s_j[0], acc_n = 0;

    // Activation fragments of the tile in each ring position: ordinary loads issued a whole
    // tile early, right after the tile's LDS-direct loads (an L2 round trip that would
    // otherwise be waited for in the open, once per tile).  A step starts by waiting for
    // everything in flight, which is its own tile and fragments and nothing else: the
    // compiler's own wait for the fragments, which cannot count the LDS-direct loads, then
    // lands where nothing newer is outstanding.  The price is 8 MT more live registers, which
    // is why MT = 2 runs with two waves per SIMD (seven streaming waves).
    static_assert(MT == 1 || (MT == 2 && WAVES <= 7), "register budget: 168 per lane above eight waves");
    u32x4 afrag[2][2][MT];
    auto load_fragments = [&](int d, uint32_t kb) {
        const uint8_t *src = reinterpret_cast<const uint8_t *>(A + (size_t)kb * 64);
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < MT; ++j) afrag[d][kh][j] = *reinterpret_cast<const u32x4 *>(src + rowoff[j] + 64 * kh);
    };
    load_fragments(0, s_kb[0]);

    // One iteration decodes the tile in ring position CUR while position CUR ^ 1 is refilled.
    auto step = [&](auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        ZS_T(0)
        wait_dma<0>(); // tile CUR, its L window and its fragments have landed
        ZS_T(6)
        lds_fence();   // all LDS reads of the slot to refill are done
        take_finish(); // (waits for the scalar loads of the offset pairs, issued a tile ago)
        // the bit-plane bytes of tile CUR are read while the next tile is staged
        BlockIndex bi;
        index_read_planes(ring + CUR * S::kBytes + S::kPlanes, lane, bi);
        u32x4 bfrag[2][MT];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                asm volatile("" : "+v"(afrag[CUR][kh][j])); // the compiler's wait for them goes here
                bfrag[kh][j] = afrag[CUR][kh][j];
            }
        {
            const uint32_t slot_at = ring + NXT * S::kBytes;
            const uint8_t *planes = bv.bitmaps + (size_t)(p_valid ? p_g : 0u) * ZS_BT_BITMAP_BYTES;
            take_begin();
            if (p_valid && p_sg.h_room >= 256u) {
                const uint32_t n3 = min(max(p_sg.h_bytes >> 4, 193u) - 192u, 64u); // lanes of the last H chunk
                stage_fast6(lane * 16, slot_at, planes, p_sg.h, ~0ull >> (64u - n3));
            } else {
                dma_segment<2>(planes, p_valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane * 16, bv.bitmaps);
                dma_segment<4>(p_sg.h, p_sg.h_bytes, slot_at + S::kH, lane * 16, bv.bitmaps);
            }
            dma_segment<S::kLChunks>(p_sg.l, min(p_sg.l_bytes, (uint32_t)LW), slot_at + S::kL, lane * 16, bv.bitmaps);
            load_fragments(NXT, p_valid ? p_kb : 0u);
            note(NXT);
        }
        ZS_T(1)
        take_lookup();
        ZS_T(2)
        if (s_j[CUR] != acc_j) {
            flush(acc_j, acc_n);
            clear_acc();
            acc_j = s_j[CUR], acc_n = 0;
        }
        const uint32_t slot = ring + CUR * S::kBytes;
        index_block_tile(slot + S::kH, slot + S::kL, lane, bi);
        ZS_T(3)
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(s_l[CUR]), s_big[CUR]};
        bf16x8 bop[2][MT];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                bop[kh][j] = __builtin_bit_cast(bf16x8, bfrag[kh][j]);
            }
        auto run = [&](auto careful) {
            decode_block_tile<BASE_M1, decltype(careful)::value, true>(tab, bi, fs, [&](int tt, const u32x4 &w) {
                const bf16x8 wop = __builtin_bit_cast(bf16x8, w);
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[tt & 3][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, bop[tt >> 2][j], acc[tt & 3][j], 0, 0, 0);
            });
        };
        // rows with three or more fallbacks (or an over-long L segment) take the careful variant
        if (fs.from_global || __builtin_amdgcn_ballot_w64(bi.min_cnt < 6) != 0)
            run(std::true_type{});
        else
            run(std::false_type{});
        ++acc_n;
        ZS_T(4)
    };
    for (;;) {
        if (!s_valid[0]) break;
        step(std::integral_constant<int, 0>{});
        if (!s_valid[1]) break;
        step(std::integral_constant<int, 1>{});
    }
    if (acc_n) flush(acc_j, acc_n);
    wait_dma<0>();
#ifdef ZS_DBG_TIMING
    if (blockIdx.x == 3 && wave == 1 && lane == 0) {
        uint64_t *o = dbg;
        zs_t[9] = __builtin_readcyclecounter();
        for (int i = 0; i < 12; ++i) o[i] = zs_t[i];
        o[12] = zs_t[7] - zs_entry;
    }
#endif
}

// --------------------------------------------------------------------------------------
// ZipGEMM, wider M (up to 64 MT tokens per launch): producer and consumer waves.
//
// The decode cost of a BlockTile does not depend on M, so for more than a few tokens it is
// paid once per workgroup and shared: P producer waves stream and decode BlockTiles exactly
// as above but write the decoded weights, already in MFMA A-operand lane order, to a ring of
// R dense tiles in LDS (8 KB each); up to Q consumer waves, each owning 16 MT tokens,
// read every dense tile and run the MFMAs against their own activation fragments.  A token
// belongs to one consumer, so nothing is reduced across waves: a consumer stores (whole
// strip) or atomically adds (strip shared between workgroups) its registers when the strip
// changes.  Consumers issue no LDS-direct loads, so their global loads and stores are ordinary
// compiler-tracked ones.
//
// Work split and tile hand-out are those of gemm_stream_kernel.  Tile i of the workgroup's
// range lives in dense slot i % R.  ready[slot] = i + 1 once tile i is complete in LDS;
// consumed[slot] counts consumer passes over the slot.  A producer may write tile i when
// consumed[slot] has reached q_active * (i / R); a consumer reads tile i when ready[slot] is
// i + 1.  Every wait points to a strictly smaller tile index and tiles are handed out in
// order, so the smallest unfinished tile can always complete.
// --------------------------------------------------------------------------------------
enum : uint32_t { kPcNext = 0, kPcReady = 64, kPcConsumed = 128, kPcCtlBytes = 192, kDenseBytes = 8192 };

template <int MT, int LW, int P, int R, int Q, bool BASE_M1>
__global__ __launch_bounds__(64 * (P + Q)) void gemm_pc_kernel(BlobView bv, const uint16_t *A, int64_t lda,
                                                                          float *C, int64_t ldc, int M, int q_active)
{
    static_assert(R >= P && R <= 16, "ready / consumed words are laid out for at most 16 dense slots");
    using S = Slot<LW>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables(smem, bv.base_exp);

    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = dynamic_lds_base();
    const uint32_t ctl = tab + kTableBytes, dense0 = ctl + kPcCtlBytes;
    const uint32_t m_lane = lane & 15u, kgrp = lane >> 4;

    const uint32_t k_blocks = (uint32_t)bv.k_blocks, total = (uint32_t)bv.strips * k_blocks;
    const uint32_t g0 = (uint32_t)((uint64_t)total * blockIdx.x / gridDim.x);
    const uint32_t g1 = (uint32_t)((uint64_t)total * (blockIdx.x + 1) / gridDim.x);

    for (uint32_t i = threadIdx.x; i < kPcCtlBytes / 4; i += blockDim.x) *((LdsU32)(ctl + 4 * i)) = i == kPcNext / 4 ? g0 : 0u;
    __syncthreads();
    if (g0 >= g1) return;
    const uint32_t n_tiles = g1 - g0;

    if (wave >= (uint32_t)P) {
        // ------------------------------------------------------------------ consumer
        const uint32_t c = wave - P;
        if ((int)c >= q_active) return;
        const uint32_t tok0 = c * 16u * MT;
        // B operand of the 16x16x32 MFMA: lane l holds token l % 16 and the 8 consecutive k that
        // start at 8 * (l / 16).  Tokens >= M read token 0 instead (their columns are never stored).
        uint32_t rowoff[MT];
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const uint32_t m = tok0 + j * 16 + m_lane;
            rowoff[j] = ((int)m < M ? m : 0u) * (uint32_t)lda * 2u + kgrp * 16u;
        }
        const uint8_t *a_bytes = reinterpret_cast<const uint8_t *>(A);
        // The activation fragments are requested D tiles ahead: an L2 hit costs about as much
        // time as several tiles' worth of MFMAs.
        constexpr int D = MT == 1 ? 4 : MT == 2 ? 2 : 1;
        u32x4 frag[D][2][MT];
        auto load_frags = [&](int d, uint32_t kb) {
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    frag[d][kh][j] = *reinterpret_cast<const u32x4 *>(a_bytes + (size_t)kb * 128 + kh * 64 + rowoff[j]);
        };
        f32x4 acc[4][MT];
        auto clear_acc = [&]() {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        };
        clear_acc();
        const uint32_t strip0 = g0 / k_blocks;
        uint32_t strip = strip0, kb = g0 - strip0 * k_blocks; // of the tile being consumed
        uint32_t kb_ahead = kb;                               // of the tile whose fragments are requested next
        uint32_t in_strip = 0;                                // tiles of the current strip consumed so far
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if ((uint32_t)d < n_tiles) load_frags(d, kb_ahead);
            kb_ahead = kb_ahead + 1 == k_blocks ? 0u : kb_ahead + 1;
        }
        uint32_t slot = 0, i = 0;
        // MT = 1: the decoded weights of tile i + 1 are read into a second register set while tile
        // i is multiplied.  Wider consumers need those registers for accumulators and fragments
        // and read each operand right before its MFMAs.
        constexpr bool kPipe = MT == 1;
        u32x4 wreg[kPipe ? 2 : 1][8];
        auto wait_ready = [&](uint32_t tile, uint32_t sl) {
            while (uniform(lds_poll(ctl + kPcReady + 4 * sl)) != tile + 1) __builtin_amdgcn_s_sleep(1);
            lds_fence();
        };
        auto read_weights = [&](int p, uint32_t sl) {
            const uint32_t at = dense0 + sl * kDenseBytes + lane * 16;
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) wreg[p][tt] = *((const __attribute__((address_space(3))) u32x4 *)(at + tt * 1024));
        };
        auto hand_back = [&](uint32_t sl) {
            lds_fence(); // the slot's data is in registers
            if (lane == 0)
                __hip_atomic_fetch_add((LdsU32)(ctl + kPcConsumed + 4 * sl), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        if constexpr (kPipe) {
            wait_ready(0, 0);
            read_weights(0, 0);
        }
        auto consume = [&](auto d_c, auto p_c) {
            constexpr int d = decltype(d_c)::value, p = kPipe ? decltype(p_c)::value : 0;
            bf16x8 bop[2][MT];
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j) {
                    bop[kh][j] = __builtin_bit_cast(bf16x8, frag[d][kh][j]);
                }
            if (i + D < n_tiles) load_frags(d, kb_ahead);
            kb_ahead = kb_ahead + 1 == k_blocks ? 0u : kb_ahead + 1;
            const uint32_t slot_next = slot + 1 == (uint32_t)R ? 0u : slot + 1;
            if constexpr (kPipe) {
                hand_back(slot); // tile i was read during the previous step
                if (i + 1 < n_tiles) {
                    wait_ready(i + 1, slot_next);
                    read_weights(p ^ 1, slot_next);
                }
            } else {
                wait_ready(i, slot);
            }
            const uint32_t at = dense0 + slot * kDenseBytes + lane * 16;
#pragma unroll
            for (int tt = 0; tt < 8; ++tt) {
                const u32x4 w = kPipe ? wreg[p][tt] : *((const __attribute__((address_space(3))) u32x4 *)(at + tt * 1024));
                const bf16x8 wop = __builtin_bit_cast(bf16x8, w);
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[tt & 3][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, bop[tt >> 2][j], acc[tt & 3][j], 0, 0, 0);
            }
            if constexpr (!kPipe) hand_back(slot);
            ++in_strip;
            const bool last_of_strip = kb + 1 == k_blocks;
            if (last_of_strip || i + 1 == n_tiles) {
                // D layout of the 16x16 MFMA: a lane holds token lane % 16 and rows 4 * (lane / 16) .. + 3
                const bool whole = in_strip == k_blocks;
#pragma unroll
                for (int j = 0; j < MT; ++j) {
                    const uint32_t m = tok0 + j * 16 + m_lane;
                    if ((int)m < M) {
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb) {
                            float *dst = C + (int64_t)m * ldc + (int64_t)strip * 64 + rb * 16 + 4 * kgrp;
                            if (whole) {
                                *reinterpret_cast<f32x4 *>(dst) = acc[rb][j];
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dst + e, acc[rb][j][e]);
                            }
                        }
                    }
                }
                clear_acc();
                in_strip = 0;
                ++strip;
            }
            kb = last_of_strip ? 0u : kb + 1;
            slot = slot_next;
            ++i;
        };
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        for (;;) {
            if (i >= n_tiles) break;
            consume(I0{}, I0{});
            if constexpr (D > 1) {
                if (i >= n_tiles) break;
                consume(I1{}, I1{});
            }
            if constexpr (D > 2) {
                if (i >= n_tiles) break;
                consume(I2{}, I0{});
                if (i >= n_tiles) break;
                consume(I3{}, I1{});
            }
        }
        return;
    }

    // ---------------------------------------------------------------------- producer
    const uint32_t ring = dense0 + R * kDenseBytes + wave * (2 * S::kBytes);
    bool p_valid = false;
    uint32_t p_g = 0;
    Segments p_sg = {bv.H, bv.L, 0u, 0u, 0u, 0u};
    uint32_t g_taken = 0;
    OffsetPairs p_off = {u32x2{0u, 0u}, u32x2{0u, 0u}};
    auto take_begin = [&]() {
        g_taken = 0;
        if (lane == 0)
            g_taken = __hip_atomic_fetch_add((LdsU32)(ctl + kPcNext), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto take_lookup = [&]() {
        const uint32_t g = uniform(g_taken);
        p_valid = g < g1;
        if (p_valid) {
            p_g = g;
            p_off = offset_pairs(bv, g);
        }
    };
    auto take_finish = [&]() {
        p_sg = Segments{bv.H, bv.L, 0u, 0u, 0u, 0u};
        if (p_valid) p_sg = segments_from(bv, p_off);
    };
    bool s_valid[2] = {false, false};
    uint32_t s_i[2] = {0u, 0u};
    const uint8_t *s_l[2] = {bv.L, bv.L};
    bool s_big[2] = {false, false};
    // Issues the Slot::kLoads LDS-direct loads of the pending tile into ring position d.
    auto stage = [&](int d) {
        const uint32_t slot_at = ring + d * S::kBytes;
        const uint8_t *planes = bv.bitmaps + (size_t)(p_valid ? p_g : 0u) * ZS_BT_BITMAP_BYTES;
        if (p_valid && p_sg.h_room >= 256u) {
            const uint32_t n3 = min(max(p_sg.h_bytes >> 4, 193u) - 192u, 64u); // lanes of the last H chunk
            stage_fast6(lane * 16, slot_at, planes, p_sg.h, ~0ull >> (64u - n3));
        } else {
            dma_segment<2>(planes, p_valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane * 16, bv.bitmaps);
            dma_segment<4>(p_sg.h, p_sg.h_bytes, slot_at + S::kH, lane * 16, bv.bitmaps);
        }
        dma_segment<S::kLChunks>(p_sg.l, min(p_sg.l_bytes, (uint32_t)LW), slot_at + S::kL, lane * 16, bv.bitmaps);
        s_valid[d] = p_valid, s_i[d] = p_g - g0, s_l[d] = p_sg.l, s_big[d] = p_sg.l_bytes > (uint32_t)LW;
    };

    take_begin();
    take_lookup();
    take_finish();
    stage(0);
    take_begin();
    take_lookup();

    auto step = [&](auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        lds_fence(); // all LDS reads of the slot to refill are done
        take_finish();
        stage(NXT);
        take_begin();
        wait_dma<S::kLoads>(); // everything older than the tile just staged has landed
        take_lookup();

        const uint32_t slot = ring + CUR * S::kBytes;
        BlockIndex bi;
        index_read_planes(slot + S::kPlanes, lane, bi);
        index_block_tile(slot + S::kH, slot + S::kL, lane, bi);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(s_l[CUR]), s_big[CUR]};

        // the dense slot must have been read by every consumer before it is overwritten
        const uint32_t i = s_i[CUR], dslot = i % (uint32_t)R, need = (uint32_t)q_active * (i / (uint32_t)R);
        while ((int32_t)(uniform(lds_poll(ctl + kPcConsumed + 4 * dslot)) - need) < 0) __builtin_amdgcn_s_sleep(1);
        const uint32_t out = dense0 + dslot * kDenseBytes + lane * 16;
        auto run = [&](auto careful) {
            decode_block_tile<BASE_M1, decltype(careful)::value, true>(tab, bi, fs, [&](int tt, const u32x4 &w) {
                *((__attribute__((address_space(3))) u32x4 *)(out + tt * 1024)) = w;
            });
        };
        // rows with three or more fallbacks (or an over-long L segment) take the careful variant
        if (fs.from_global || __builtin_amdgcn_ballot_w64(bi.min_cnt < 6) != 0)
            run(std::true_type{});
        else
            run(std::false_type{});
        lds_fence(); // the tile is complete in LDS before it is announced
        if (lane == 0)
            __hip_atomic_store((LdsU32)(ctl + kPcReady + 4 * dslot), i + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    for (;;) {
        if (!s_valid[0]) break;
        step(std::integral_constant<int, 0>{});
        if (!s_valid[1]) break;
        step(std::integral_constant<int, 1>{});
    }
    wait_dma<0>();
}

// Clears the columns of C that belong to strips shared by several workgroups of the ZipGEMM
// launch that follows (they are summed with atomics).  The host lists those strips (a range
// boundary that is not a multiple of k_blocks cuts exactly one strip, so there are fewer than
// the number of workgroups); the list travels in the kernel arguments.  One workgroup per
// listed strip.
constexpr int kMaxSharedStrips = 512;
struct SharedStrips {
    uint32_t n;
    uint32_t strip[kMaxSharedStrips];
};

__global__ void clear_shared_strips_kernel(float *C, int64_t ldc, int M, SharedStrips list)
{
    const uint32_t strip = list.strip[blockIdx.x];
    for (uint32_t i = threadIdx.x; i < (uint32_t)M * 16u; i += blockDim.x) {
        const uint32_t m = i >> 4, c = i & 15u;
        *reinterpret_cast<f32x4 *>(C + (int64_t)m * ldc + (int64_t)strip * 64 + 4 * c) = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// --------------------------------------------------------------------------------------
// Host side
// --------------------------------------------------------------------------------------
int make_view(const zs_desc *d, const void *blob, BlobView *bv)
{
    if (!d || !blob) return ZS_ERR_ARG;
    int rc = zs_desc_validate(d);
    if (rc != ZS_OK) return rc;
    if (reinterpret_cast<uintptr_t>(blob) % ZS_SECTION_ALIGN) return ZS_ERR_ARG;
    if ((uint64_t)(d->N / 64) * (uint64_t)(d->K / 64) >= (1ull << 31)) return ZS_ERR_SHAPE;
    const uint8_t *b = static_cast<const uint8_t *>(blob);
    bv->bitmaps = b + d->off_bitmaps;
    bv->offsets = reinterpret_cast<const u32x2 *>(b + d->off_offsets);
    bv->H = b + d->off_H;
    bv->L = b + d->off_L;
    bv->h_units = (uint32_t)(d->h_bytes / 16);
    bv->l_units = (uint32_t)(d->l_bytes / 16);
    bv->base_exp = d->base_exp;
    bv->k_blocks = (int32_t)(d->K / 64);
    bv->strips = (int32_t)(d->N / 64);
    return ZS_OK;
}

template <class Kernel>
int allow_big_lds(Kernel k, uint32_t bytes)
{
    if (bytes > kMaxLds) return ZS_ERR_CONFIG;
    if (bytes > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) !=
            hipSuccess)
        return ZS_ERR_HIP;
    return ZS_OK;
}

// Window of the L segment staged in LDS, in bytes: twice the average BlockTile's segment
// (BlockTiles with more take their fallbacks from global memory).
int pick_l_window(const zs_desc *d)
{
    const uint64_t n_bt = (uint64_t)(d->N / 64) * (uint64_t)(d->K / 64);
    const uint64_t avg = 2 * d->n_fallback / n_bt; // bytes per BlockTile
    const uint64_t want = d->max_l_units * 16ull < 2 * avg ? d->max_l_units * 16ull : 2 * avg;
    return want <= 512 ? 512 : 4096;
}

struct GemmVariant {
    const char *name;
    int mt, lw, waves;
    int consumers; // 0: gemm_stream_kernel (16 mt tokens); else gemm_pc_kernel with that many consumer waves
    bool shared_decode() const { return consumers > 0; }
    int tokens() const { return 16 * mt * (consumers ? consumers : 1); }
};

// id = index + 1.  The first entry of each (tokens, lw) pair is the default for that pair.
// Names: m<tokens per launch>_l<0: 512-byte, 4: 4 KB L window>_w<streaming waves> for
// gemm_stream_kernel, p<tokens per launch>_l<..>_w<producer waves> for gemm_pc_kernel.
const GemmVariant kVariants[] = {
    {"m16_l0_w11", 1, 512, 11, 0}, {"m16_l0_w8", 1, 512, 8, 0},   {"m32_l0_w7", 2, 512, 7, 0},
    {"m32_l0_w6", 2, 512, 6, 0},   {"m16_l4_w7", 1, 4096, 7, 0},  {"m32_l4_w6", 2, 4096, 6, 0},
    {"p64_l0_w7", 1, 512, 7, 4},   {"p128_l0_w7", 2, 512, 7, 4},  {"p256_l0_w7", 2, 512, 7, 8},
    {"p64_l4_w5", 1, 4096, 5, 4},  {"p128_l4_w5", 2, 4096, 5, 4}, {"p256_l4_w5", 2, 4096, 5, 8},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

// Workgroups of a ZipGEMM launch: one per CU, fewer when there are fewer BlockTiles.
uint32_t auto_workgroups(const BlobView &bv)
{
    const uint64_t total = (uint64_t)bv.strips * (uint64_t)bv.k_blocks;
    return (uint32_t)(total < (uint64_t)kNumCus ? total : (uint64_t)kNumCus);
}

// C must start from zero where some workgroup's range begins or ends inside a strip: those
// strips are summed from several workgroups with atomics.
void clear_shared_strips(const BlobView &bv, float *C, int64_t ldc, int M, uint32_t wgs, hipStream_t s)
{
    const uint64_t total = (uint64_t)bv.strips * (uint64_t)bv.k_blocks;
    SharedStrips list;
    list.n = 0;
    for (uint32_t b = 1; b < wgs; ++b) {
        const uint64_t g = total * b / wgs;
        if (g % (uint64_t)bv.k_blocks == 0) continue;
        const uint32_t strip = (uint32_t)(g / (uint64_t)bv.k_blocks);
        if (list.n && list.strip[list.n - 1] == strip) continue; // boundaries ascend: duplicates are adjacent
        list.strip[list.n++] = strip;
        if (list.n == (uint32_t)kMaxSharedStrips) { // flush a full list
            hipLaunchKernelGGL(clear_shared_strips_kernel, dim3(list.n), dim3(256), 0, s, C, ldc, M, list);
            list.n = 0;
        }
    }
    if (list.n) hipLaunchKernelGGL(clear_shared_strips_kernel, dim3(list.n), dim3(256), 0, s, C, ldc, M, list);
}

// Layout of the scratch buffer of gemm_stream_kernel: kMaxSharedCounters counter words (zero
// between launches), then two partial tiles of 4096 MT bytes per workgroup.  The counter area
// has one size for every matrix and configuration, so that a buffer which served one call
// has zero counters for any other.
constexpr uint32_t kMaxSharedCounters = 1024;
size_t shared_sums_bytes(uint32_t wgs, int mt) { return kMaxSharedCounters * 4 + (size_t)2 * wgs * 4096 * (size_t)mt; }

template <int MT, int LW, int WAVES>
int launch_gemm(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, uint32_t wgs,
                void *scratch, uint64_t *dbg, hipStream_t s)
{
    using S = Slot<LW>;
    constexpr uint32_t lds = kTableBytes + 2 * 16 * 16 * MT * 16 + kCtlBytes + WAVES * 2 * S::kBytes;
    static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
    static_assert(S::kLoads < 64, "vmcnt cannot count that many loads");
    const bool m1 = bv.base_exp < 0;
    auto kern = m1 ? gemm_stream_kernel<MT, LW, WAVES, true> : gemm_stream_kernel<MT, LW, WAVES, false>;
    int rc = allow_big_lds(kern, lds);
    if (rc != ZS_OK) return rc;
    SharedSums ws = {nullptr, nullptr};
    if (scratch) {
        ws.count = static_cast<uint32_t *>(scratch);
        ws.tiles = reinterpret_cast<float *>(static_cast<uint8_t *>(scratch) + kMaxSharedCounters * 4);
    } else {
        clear_shared_strips(bv, C, ldc, M, wgs, s);
    }
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(64 * (WAVES + 1)), lds, s, bv, A, lda, C, ldc, M, ws, dbg);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

template <int MT, int LW, int P, int R, int Q>
int launch_pc(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, uint32_t wgs,
              hipStream_t s)
{
    using S = Slot<LW>;
    constexpr uint32_t lds = kTableBytes + kPcCtlBytes + R * kDenseBytes + P * 2 * S::kBytes;
    static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
    static_assert(S::kLoads < 64, "vmcnt cannot count that many loads");
    const bool m1 = bv.base_exp < 0;
    auto kern = m1 ? gemm_pc_kernel<MT, LW, P, R, Q, true> : gemm_pc_kernel<MT, LW, P, R, Q, false>;
    int rc = allow_big_lds(kern, lds);
    if (rc != ZS_OK) return rc;
    clear_shared_strips(bv, C, ldc, M, wgs, s);
    const int q_active = ((M + 15) / 16 + MT - 1) / MT; // consumers with at least one token
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(64 * (P + Q)), lds, s, bv, A, lda, C, ldc, M, q_active);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

int variant_for(const zs_desc *d, int64_t M)
{
    // up to 32 tokens every wave decodes and multiplies for itself; beyond, the decode is shared
    const int lw = pick_l_window(d);
    const int tokens = M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : M <= 128 ? 128 : 256;
    const bool shared_decode = tokens > 32;
    // Waves take BlockTiles one at a time, so a workgroup's last round is rarely full.  With few
    // tiles per workgroup eight waves (faster each, fuller rounds) beat eleven; measured on the
    // 8B shapes the crossover lies between 56 and 112 tiles per workgroup.
    const int64_t tiles_per_wg = (d->N / 64) * (d->K / 64) / kNumCus;
    const int waves = tokens == 16 && lw == 512 && tiles_per_wg <= 64 ? 8 : 0;
    for (int i = 0; waves && i < kNumVariants; ++i)
        if (kVariants[i].tokens() == tokens && kVariants[i].lw == lw && !kVariants[i].shared_decode() &&
            kVariants[i].waves == waves)
            return i + 1;
    for (int i = 0; i < kNumVariants; ++i)
        if (kVariants[i].tokens() == tokens && kVariants[i].lw == lw && kVariants[i].shared_decode() == shared_decode)
            return i + 1;
    return 1;
}

} // namespace

extern "C" int zs_decompress(const zs_desc *d, const void *blob_dev, uint16_t *W_out_dev, int64_t ldw,
                             void *hip_stream)
{
    BlobView bv;
    int rc = make_view(d, blob_dev, &bv);
    if (rc != ZS_OK) return rc;
    if (!W_out_dev || reinterpret_cast<uintptr_t>(W_out_dev) % 16) return ZS_ERR_ARG;
    if (ldw < d->K || ldw % 8) return ZS_ERR_SHAPE;
    const int64_t n_bt = (int64_t)bv.strips * bv.k_blocks;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    auto launch = [&](auto kern, uint32_t lds, int waves) {
        int r = allow_big_lds(kern, lds);
        if (r != ZS_OK) return r;
        int64_t wgs = (n_bt + waves - 1) / waves;
        if (wgs > kNumCus) wgs = kNumCus;
        hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(64 * waves), lds, s, bv, W_out_dev, ldw);
        return hipGetLastError() == hipSuccess ? (int)ZS_OK : (int)ZS_ERR_HIP;
    };
    const bool m1 = d->base_exp < 0;
    if (pick_l_window(d) == 512) {
        constexpr uint32_t lds = kTableBytes + 7 * 3 * Slot<1024>::kBytes;
        return m1 ? launch(decompress_kernel<1024, 3, 7, true>, lds, 7)
                  : launch(decompress_kernel<1024, 3, 7, false>, lds, 7);
    }
    constexpr uint32_t lds = kTableBytes + 7 * 2 * Slot<4096>::kBytes;
    return m1 ? launch(decompress_kernel<4096, 2, 7, true>, lds, 7) : launch(decompress_kernel<4096, 2, 7, false>, lds, 7);
}

extern "C" int zs_gemm_num_configs(void) { return kNumVariants; }

extern "C" const char *zs_gemm_config_name(int config)
{
    return (config >= 1 && config <= kNumVariants) ? kVariants[config - 1].name : nullptr;
}

extern "C" int zs_gemm_pick_config(const zs_desc *d, int64_t M)
{
    if (!d || M < 1 || zs_desc_validate(d) != ZS_OK) return 0;
    return variant_for(d, M);
}

extern "C" size_t zs_gemm_workspace_ex(const zs_desc *d, int64_t M, int config)
{
    if (!d || M < 1 || config < 0 || zs_desc_validate(d) != ZS_OK) return 0;
    int variant = config & 0xFF;
    if (variant == 0) variant = variant_for(d, M);
    if (variant < 1 || variant > kNumVariants) return 0;
    const GemmVariant &v = kVariants[variant - 1];
    if (v.shared_decode()) return 0; // the producer / consumer kernel sums shared strips with atomics on C
    BlobView bv;
    bv.strips = (int32_t)(d->N / 64), bv.k_blocks = (int32_t)(d->K / 64);
    const uint64_t total = (uint64_t)bv.strips * (uint64_t)bv.k_blocks;
    uint32_t wgs = (uint32_t)(config >> 8);
    if (wgs == 0) wgs = auto_workgroups(bv);
    if (wgs > total) wgs = (uint32_t)total;
    return wgs <= kMaxSharedCounters ? shared_sums_bytes(wgs, v.mt) : 0;
}
extern "C" size_t zs_gemm_workspace(const zs_desc *d, int64_t M) { return zs_gemm_workspace_ex(d, M, 0); }

extern "C" int zs_gemm_ex(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                          int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream,
                          int config)
{
    BlobView bv;
    int rc = make_view(d, blob_dev, &bv);
    if (rc != ZS_OK) return rc;
    if (!A_dev || !C_dev) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(A_dev) % 16 || reinterpret_cast<uintptr_t>(C_dev) % 16) return ZS_ERR_ARG;
    if (M < 1 || M > (1 << 20) || lda < d->K || lda % 8 || ldc < d->N || ldc % 4) return ZS_ERR_SHAPE;
    if (config < 0) return ZS_ERR_CONFIG;
    int variant = config & 0xFF;
    if (variant == 0) variant = variant_for(d, M);
    if (variant < 1 || variant > kNumVariants) return ZS_ERR_CONFIG;
    const GemmVariant &v = kVariants[variant - 1];
    // bits 8 and up of config: number of workgroups (0 = one per CU)
    uint32_t wgs = (uint32_t)(config >> 8);
    const uint64_t total = (uint64_t)bv.strips * (uint64_t)bv.k_blocks;
    if (wgs == 0) wgs = auto_workgroups(bv);
    if (wgs > total) wgs = (uint32_t)total;
    if ((uint64_t)lda * 2u * 64u >= (1ull << 32)) return ZS_ERR_SHAPE; // row offsets are 32-bit inside the kernel
    uint64_t *dbg = nullptr;
    void *scratch = nullptr;
#ifdef ZS_DBG_TIMING
    (void)workspace_bytes;
    dbg = static_cast<uint64_t *>(workspace_dev); // debug builds dump their cycle counts here
#else
    // scratch is optional: without it (or with too little) shared strips go through atomics on C
    if (workspace_dev && !v.shared_decode() && reinterpret_cast<uintptr_t>(workspace_dev) % 256 == 0 &&
        wgs <= kMaxSharedCounters && workspace_bytes >= shared_sums_bytes(wgs, v.mt))
        scratch = workspace_dev;
#endif
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // tokens beyond the variant's width are handled in successive column panels
    const int width = v.tokens();
    for (int64_t m0 = 0; m0 < M; m0 += width) {
        const int m = (int)((M - m0) < width ? (M - m0) : width);
        const uint16_t *Ap = A_dev + m0 * lda;
        float *Cp = C_dev + m0 * ldc;
#define ZS_PC_CASE(ID, MT, LW, P, R, Q) \
    case ID: rc = launch_pc<MT, LW, P, R, Q>(bv, Ap, lda, Cp, ldc, m, wgs, s); break;
#define ZS_CASE(ID, MT, LW, WAVES) \
    case ID: rc = launch_gemm<MT, LW, WAVES>(bv, Ap, lda, Cp, ldc, m, wgs, scratch, dbg, s); break;
        switch (variant) {
            ZS_CASE(1, 1, 512, 11)
            ZS_CASE(2, 1, 512, 8)
            ZS_CASE(3, 2, 512, 7)
            ZS_CASE(4, 2, 512, 6)
            ZS_CASE(5, 1, 4096, 7)
            ZS_CASE(6, 2, 4096, 6)
            ZS_PC_CASE(7, 1, 512, 7, 7, 4)
            ZS_PC_CASE(8, 2, 512, 7, 7, 4)
            ZS_PC_CASE(9, 2, 512, 7, 7, 8)
            ZS_PC_CASE(10, 1, 4096, 5, 5, 4)
            ZS_PC_CASE(11, 2, 4096, 5, 5, 4)
            ZS_PC_CASE(12, 2, 4096, 5, 5, 8)
        default: rc = ZS_ERR_CONFIG;
        }
#undef ZS_CASE
#undef ZS_PC_CASE
        if (rc != ZS_OK) return rc;
    }
    return ZS_OK;
}

extern "C" int zs_gemm(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                       int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    return zs_gemm_ex(d, blob_dev, A_dev, lda, C_dev, ldc, M, workspace_dev, workspace_bytes, hip_stream, 0);
}

extern "C" const char *zs_strerror(int status)
{
    switch (status) {
    case ZS_OK: return "ok";
    case ZS_ERR_ARG: return "bad argument (null or misaligned pointer)";
    case ZS_ERR_SHAPE: return "unsupported shape (N, K must be positive multiples of 64; check M, ld*)";
    case ZS_ERR_SIZE: return "buffer too small";
    case ZS_ERR_FORMAT: return "descriptor does not describe a valid TCA-TBE blob";
    case ZS_ERR_HIP: return "HIP runtime error";
    case ZS_ERR_CONFIG: return "unknown kernel configuration";
    default: return "unknown status";
    }
}

extern "C" int zs_version(void) { return 1; }
