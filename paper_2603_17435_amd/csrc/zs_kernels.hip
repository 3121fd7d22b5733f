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

#include <atomic>
#include <cstring>
#include <type_traits>

#include "zipserv.h"
#include "zs_device.h"

using namespace zs;


namespace {

constexpr uint32_t kMaxLds = 160 * 1024;
constexpr int kMaxDevices = 64;

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
    // what the LDS-direct loads of a tile can write: 1536 bytes of bit-planes, four 1 KB pieces of
    // H, kLChunks pieces of L (one 512-byte piece for LW = 512); all of it lies inside the slot
    static_assert(kPlanes + ZS_BT_BITMAP_BYTES <= kH && kH + 4 * 1024 <= kL, "sections of a slot overlap");
    static_assert(kL + (LW == 512 ? 512 : kLChunks * 1024) <= kBytes, "the staged L window leaves the slot");
};

// LDS image of a gemm_stream_kernel workgroup, shared by the kernel (addresses) and the host
// (bytes to request): tables | two accumulation tiles | control words | WAVES rings of kDepth slots.
template <int MT, int LW, int WAVES>
struct StreamLds {
    static constexpr uint32_t kDepth = 2; // ring positions per wave: one tile decoded, one in flight
    static constexpr uint32_t kUnits = 16 * MT * 16, kTileBytes = 16 * kUnits; // float4 units of an accumulation tile
    static constexpr uint32_t kRed = kTableBytes, kCtl = kRed + 2 * kTileBytes, kRings = kCtl + 64;
    static constexpr uint32_t kTotal = kRings + WAVES * kDepth * Slot<LW>::kBytes;
    static_assert(kTotal <= 160 * 1024, "variant does not fit the 160 KB of LDS");
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

__device__ __forceinline__ uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

// LDS address of the dynamic shared array: it follows the kernel's static LDS (a link-time
// constant; these kernels have none).  Taking the address through a pointer cast instead
// leaves a null-pointer select at every use.
__device__ __forceinline__ uint32_t dynamic_lds_base() { return __builtin_amdgcn_groupstaticsize(); }

// All LDS-direct loads of a BlockTile whose segments start far enough from the ends of their
// sections (BlobView::h_fast, l_fast): 1536 bytes of bit-planes, 4096 bytes from the start of
// the H segment and LW bytes from the start of the L segment, whatever the segments' lengths
// (what lies beyond them belongs to the next BlockTiles and is ignored).  No address or lane
// mask is computed: three base registers, instruction offsets, and the lower half of the wave
// for the two 512-byte pieces.  Exactly Slot<LW>::kLoads instructions; nothing is waited for.
// All operands except lane16 (= 16 * lane) are wave-uniform; all 64 lanes must be active.
template <int LW>
__device__ __forceinline__ void stage_fast(uint32_t lane16, uint32_t slot_at, const uint8_t *planes, const uint8_t *h,
                                           const uint8_t *l)
{
    using S = Slot<LW>;
    static_assert(S::kPlanes == 0 && S::kH == 1536 && S::kL == 5632, "the LDS offsets below assume this slot layout");
    static_assert(LW == 512 || LW == 1024 || LW == 4096, "L windows staged below");
#define ZS_LOAD "global_load_lds_dwordx4 %[l16], "
    if constexpr (LW == 512) {
        asm volatile("s_mov_b32 m0, %[slot]\n\ts_nop 0\n\t" ZS_LOAD "%[bp]\n\t"
                     "s_add_u32 m0, %[slot], 1536\n\ts_nop 0\n\t" ZS_LOAD "%[bh]\n\t" ZS_LOAD "%[bh] offset:1024\n\t"
                     ZS_LOAD "%[bh] offset:2048\n\t" ZS_LOAD "%[bh] offset:3072\n\t"
                     "s_mov_b32 m0, %[slot]\n\ts_mov_b64 exec, %[half]\n\t" ZS_LOAD "%[bp] offset:1024\n\t"
                     "s_add_u32 m0, %[slot], 5632\n\ts_nop 0\n\t" ZS_LOAD "%[bl]\n\t"
                     "s_mov_b64 exec, -1"
                     :
                     : [l16] "v"(lane16), [slot] "s"(slot_at), [bp] "s"(planes), [bh] "s"(h), [bl] "s"(l),
                       [half] "s"(0xFFFFFFFFull)
                     : "memory", "scc", "m0");
    } else if constexpr (LW == 1024) {
        asm volatile("s_mov_b32 m0, %[slot]\n\ts_nop 0\n\t" ZS_LOAD "%[bp]\n\t"
                     "s_add_u32 m0, %[slot], 1536\n\ts_nop 0\n\t" ZS_LOAD "%[bh]\n\t" ZS_LOAD "%[bh] offset:1024\n\t"
                     ZS_LOAD "%[bh] offset:2048\n\t" ZS_LOAD "%[bh] offset:3072\n\t"
                     "s_add_u32 m0, %[slot], 5632\n\ts_nop 0\n\t" ZS_LOAD "%[bl]\n\t"
                     "s_mov_b32 m0, %[slot]\n\ts_mov_b64 exec, %[half]\n\t" ZS_LOAD "%[bp] offset:1024\n\t"
                     "s_mov_b64 exec, -1"
                     :
                     : [l16] "v"(lane16), [slot] "s"(slot_at), [bp] "s"(planes), [bh] "s"(h), [bl] "s"(l),
                       [half] "s"(0xFFFFFFFFull)
                     : "memory", "scc", "m0");
    } else {
        asm volatile("s_mov_b32 m0, %[slot]\n\ts_nop 0\n\t" ZS_LOAD "%[bp]\n\t"
                     "s_add_u32 m0, %[slot], 1536\n\ts_nop 0\n\t" ZS_LOAD "%[bh]\n\t" ZS_LOAD "%[bh] offset:1024\n\t"
                     ZS_LOAD "%[bh] offset:2048\n\t" ZS_LOAD "%[bh] offset:3072\n\t"
                     "s_add_u32 m0, %[slot], 5632\n\ts_nop 0\n\t" ZS_LOAD "%[bl]\n\t" ZS_LOAD "%[bl] offset:1024\n\t"
                     ZS_LOAD "%[bl] offset:2048\n\t" ZS_LOAD "%[bl] offset:3072\n\t"
                     "s_mov_b32 m0, %[slot]\n\ts_mov_b64 exec, %[half]\n\t" ZS_LOAD "%[bp] offset:1024\n\t"
                     "s_mov_b64 exec, -1"
                     :
                     : [l16] "v"(lane16), [slot] "s"(slot_at), [bp] "s"(planes), [bh] "s"(h), [bl] "s"(l),
                       [half] "s"(0xFFFFFFFFull)
                     : "memory", "scc", "m0");
    }
#undef ZS_LOAD
}

// A BlockTile as the issuing side of a wave knows it (everything wave-uniform): its number and
// the two offset pairs {H start, L start} that bracket it.  "No tile" is g = kNoTileG with
// offsets of all ones (BlockTile numbers are below 2^31; the offsets then fail the bounds test
// of the common staging path).
struct TileRef {
    uint32_t g;
    u32x4 off; // {H start, L start, next H start, next L start}, 16-byte units
};
constexpr uint32_t kNoTileG = ~0u;
#define kNoTileOff (u32x4{~0u, ~0u, ~0u, ~0u})

// What the decoding side needs to know about the L segment of a staged tile.
struct StagedL {
    const uint8_t *l; // the segment in global memory
    uint32_t big;     // nonzero: it is longer than the staged window, fallbacks are read from `l`
};

// Both offset pairs of BlockTile bt with one scalar load (the offset array is read-only for the
// launch: through the constant address space a wave-uniform index becomes a scalar load, which
// does not share the vector-memory counter with the LDS-direct loads).
__device__ __forceinline__ u32x4 offset_quad(const BlobView &bv, uint32_t bt)
{
    typedef uint32_t __attribute__((ext_vector_type(4), aligned(8))) Quad;
    typedef const Quad __attribute__((address_space(4))) *ConstQuad;
    const Quad q = *(ConstQuad)(uintptr_t)(bv.offsets + bt);
    return u32x4{q.x, q.y, q.z, q.w};
}

// Stages tile t into the slot at slot_at with exactly Slot<LW>::kLoads LDS-direct instructions
// (also for "no tile": then only lane 0 runs, on a dummy address).  No read can leave the blob
// sections or the slot whatever the offset array holds: the common path checks the segment
// starts against the precomputed bounds, the other one clamps every start and length.
template <int LW>
__device__ __forceinline__ StagedL stage_tile(const BlobView &bv, const TileRef &t, uint32_t slot_at, uint32_t lane)
{
    using S = Slot<LW>;
    const uint32_t h0 = t.off.x, l0 = t.off.y;
    if (h0 < bv.h_fast && l0 < bv.l_fast) {
        const uint8_t *l = bv.L + (size_t)l0 * 16;
        stage_fast<LW>(lane * 16, slot_at, bv.bitmaps + (size_t)t.g * ZS_BT_BITMAP_BYTES, bv.H + (size_t)h0 * 16, l);
        // a wrong length can only choose the wrong source of fallbacks: both are readable
        return StagedL{l, t.off.w - l0 > (uint32_t)(LW / 16) ? 1u : 0u};
    }
    const bool valid = t.g != kNoTileG;
    Segments sg = {bv.H, bv.L, 0u, 0u, 0u, 0u};
    if (valid) sg = segments_from(bv, OffsetPairs{u32x2{t.off.x, t.off.y}, u32x2{t.off.z, t.off.w}});
    const uint8_t *planes = bv.bitmaps + (size_t)(valid ? t.g : 0u) * ZS_BT_BITMAP_BYTES;
    dma_segment<2>(planes, valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane * 16, bv.bitmaps);
    dma_segment<4>(sg.h, sg.h_bytes, slot_at + S::kH, lane * 16, bv.bitmaps);
    dma_segment<S::kLChunks>(sg.l, min(sg.l_bytes, (uint32_t)LW), slot_at + S::kL, lane * 16, bv.bitmaps);
    return StagedL{sg.l, sg.l_bytes > (uint32_t)LW ? 1u : 0u};
}

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
        const bool valid = bt < n_bt;
        stage_tile<LW>(bv, valid ? TileRef{bt, offset_quad(bv, bt)} : TileRef{kNoTileG, kNoTileOff}, ring + j * S::kBytes, lane);
    }
    uint32_t cur = 0, nxt = DEPTH - 1; // ring positions of the tile being decoded / being issued
    for (uint32_t bt = first; bt < n_bt; bt += stride) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // every LDS read of the slot about to be refilled is done
        const uint32_t ahead = bt + (DEPTH - 1) * stride;
        const bool valid = ahead < n_bt;
        stage_tile<LW>(bv, valid ? TileRef{ahead, offset_quad(bv, ahead)} : TileRef{kNoTileG, kNoTileOff},
                       ring + nxt * S::kBytes, lane);
        wait_dma<(DEPTH - 1) * S::kLoads>();

        const uint32_t slot = ring + cur * S::kBytes;
        const Segments sg = segments_of(bv, bt);
        HalfIndex h0;
        const uint32_t pa = plane_address(slot + S::kPlanes, lane);
        read_planes<0, 0, false>(pa, h0);
        uint32_t h_base = slot + S::kH;
        index_half<true>(h_base, h0);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(sg.l), sg.l_bytes > (uint32_t)LW};
        const uint32_t strip = bt / (uint32_t)bv.k_blocks, kb = bt % (uint32_t)bv.k_blocks;
        uint16_t *dst = out + ((int64_t)strip * 64 + row_in_tt) * ldw + (int64_t)kb * 64 + col_in_tt;
        decode_block_tile<BASE_M1, 0, 0>(tab, pa, h0, h_base, l_lane_of(slot + S::kH, slot + S::kL, lane), fs,
                                         [&](int tt, const u32x4 &w) {
                                             __builtin_nontemporal_store(
                                                 w, reinterpret_cast<u32x4 *>(dst + (int64_t)((tt & 3) * 16) * ldw + (tt >> 2) * 32));
                                         });
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
// in B-operand lane order, at the top of the step that uses them: before the LDS-direct loads
// of the next tile, so that the staging and the indexing cover their L2 round trip.
// --------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) uint32_t *LdsU32;
typedef __attribute__((address_space(3))) f32x4 *LdsF32x4;

__device__ __forceinline__ uint32_t lds_poll(uint32_t at)
{
    return __hip_atomic_load((LdsU32)at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Waits for every LDS and scalar-memory operation of the wave.  The builtin (not inline
// assembly) lets the compiler's own wait-count bookkeeping see the wait, so it does not wait
// again, later and for more, for a scalar load that this one already covered.
__device__ __forceinline__ void lds_fence()
{
    __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0), the other counters untouched
    asm volatile("" ::: "memory");
}

// Control words in LDS (byte offsets from the control block).
enum : uint32_t { kCtlNext = 0, kCtlWritten = 4, kCtlLock = 8, kCtlDone = 16, kCtlBytes = 64 };

// How the partial sums of a strip that several workgroups contribute to become C.
//   kSumCleared  the host cleared the strip's columns with a kernel of its own before this
//                launch; contributors add with FP32 atomics (no scratch memory needed)
//   kSumParked   contributors park their partial tiles in scratch memory and count themselves
//                in; the last one adds the tiles up and stores the strip
// count[b] belongs to the shared strip whose first contributor is workgroup b (unique: a range
// that holds the starts of two strips holds the first of them whole); it is zero between
// launches (whoever counts last takes it down).  tiles holds two slots per workgroup (for its
// first and its last task), each 64 rows x 16 MT tokens of FP32, all zero bits between
// launches as well (the last contributor clears what it has read).
// Measured and dropped: the first contributor zeroing the columns and raising a flag, everybody
// adding with atomics once the flag is up (no round trip at the end of the kernel, but the
// atomics themselves take longer than the exchange through kSumParked at 32 tokens).
enum : uint32_t { kSumCleared = 0, kSumParked = 1 };
struct SharedSums {
    uint32_t *count;
    float *tiles;
    uint32_t mode;
    uint32_t out_bf16;    // nonzero: C holds BF16 bit patterns (ldc in those elements); needs kSumParked
    uint32_t tiles_bytes; // size of the slot area at `tiles` (two slots per workgroup)
};

// FP32 -> BF16 bit pattern, round to nearest even; NaN stays NaN (quiet bit set, sign and the
// upper payload bits kept).
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? ((u >> 16) | 0x40u) : rounded;
}

// The BlockTile sequence [0, total) is cut into `parts` contiguous ranges of q or q + 1
// BlockTiles (the first r ranges have q + 1), total = parts * q + r.  The host fills the
// struct, so that no kernel divides by a run-time value on its main path.
struct RangeSplit {
    uint32_t total, parts, q, r;
    __host__ __device__ uint32_t begin(uint32_t b) const { return b * q + (b < r ? b : r); }
    // the range that BlockTile g lies in
    __host__ __device__ uint32_t of(uint32_t g) const
    {
        const uint32_t wide = r * (q + 1);
        return g < wide ? g / (q + 1) : r + (g - wide) / q;
    }
};

template <int MT, int LW, int WAVES, bool BASE_M1>
__global__ __launch_bounds__(64 * (WAVES + 1)) void gemm_stream_kernel(BlobView bv, const uint16_t *A, int64_t lda,
                                                                  float *C, int64_t ldc, int M, SharedSums ws,
                                                                  RangeSplit rs)
{
    using S = Slot<LW>;
    using Lds = StreamLds<MT, LW, WAVES>;
    constexpr int DEPTH = Lds::kDepth;
    // LDS after the tables: two accumulation tiles (16 MT tokens x 64 rows, FP32, in units of
    // float4 = 4 consecutive rows; unit (m, c) lives at m * 16 + (c ^ (m & 15)) so that the 16
    // tokens of one MFMA result hit 16 different bank groups), the control words, the rings.
    constexpr uint32_t kUnits = Lds::kUnits, kTileBytes = Lds::kTileBytes;
    static_assert(Lds::kRings == Lds::kCtl + kCtlBytes, "control block size");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = dynamic_lds_base();
    const uint32_t red = tab + Lds::kRed, ctl = tab + Lds::kCtl;
    // the last byte any wave's ring can reach is Lds::kTotal, which is what the host requests
    const uint32_t ring = tab + Lds::kRings + wave * (DEPTH * S::kBytes);
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
    const uint32_t k_blocks = (uint32_t)bv.k_blocks;
    // Workgroups are dealt out to the chip's eight dies round-robin (workgroup b runs on die
    // b % 8).  Neighbouring ranges share a strip and exchange partial tiles, so a die takes a
    // run of consecutive ranges; a bijection on [0, gridDim.x) whenever 8 divides the grid.
    const uint32_t range_id = (gridDim.x & 7u) == 0 ? (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const uint32_t g0 = rs.begin(range_id), g1 = rs.begin(range_id + 1);
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

    // ---- issuing side: takes the next BlockTile off the shared counter and looks up its offsets.
    // The counter hands out positions c = 0 .. g1 - g0 - 1 in processing order; positions below
    // rot lie in the range's last strip (task 0), the others count from g0.
    const uint32_t n_pos = g1 - g0, first_a = strip_last * k_blocks, first_b = g0 - rot;
    uint32_t it_j = rot ? 1u : 0u, it_base = strip0 * k_blocks; // task and first BlockTile of the strip the counter is in
    uint32_t p_valid = 0;                                       // the next BlockTile to issue ... (0 / 1: plain scalars)
    uint32_t p_j = 0, p_kb = 0;
    TileRef p_t = {kNoTileG, kNoTileOff};
    // Taking the next BlockTile is spread over two points of a step so that neither the LDS
    // atomic nor the scalar load is waited for where it is issued.
    uint32_t g_taken = 0; // (per lane) what the counter returned
    auto take_begin = [&]() {
        g_taken = 0;
        if (lane == 0)
            g_taken = __hip_atomic_fetch_add((LdsU32)(ctl + kCtlNext), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto take_lookup = [&]() {
        const uint32_t c = uniform(g_taken);
        p_valid = (c - n_pos) >> 31; // c < n_pos (both below 2^31), kept a number in a scalar register
        p_t = TileRef{kNoTileG, kNoTileOff};
        if (p_valid) {
            if (c < rot) { // the range's last strip, task 0
                p_t.g = first_a + c, p_j = 0, p_kb = c;
            } else {
                const uint32_t g = first_b + c;
                while (g - it_base >= k_blocks) it_base += k_blocks, ++it_j;
                p_t.g = g, p_j = it_j, p_kb = g - it_base;
            }
            p_t.off = offset_quad(bv, p_t.g);
        }
    };
    // what the decoding side needs to know about a staged tile, per ring position (wave-uniform)
    uint32_t s_valid[DEPTH], s_j[DEPTH], s_kb[DEPTH];
    StagedL s_l[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) s_valid[d] = 0, s_j[d] = 0, s_kb[d] = 0, s_l[d] = StagedL{bv.L, 0u};
    // Issues the LDS-direct loads of the pending tile into ring position d.
    auto stage = [&](int d) {
        s_l[d] = stage_tile<LW>(bv, p_t, ring + d * S::kBytes, lane);
        s_valid[d] = p_valid, s_j[d] = p_j, s_kb[d] = p_valid ? p_kb : 0u;
    };

    // The first BlockTile of every streaming wave is assigned statically (position = wave) and
    // staged before anything else: its loads are in flight while the tables are built.
    if (wave < WAVES) {
        g_taken = wave;
        take_lookup();
        stage(0);
    }
    build_tables(smem, bv.base_exp);
    for (uint32_t i = threadIdx.x; i < (2 * kTileBytes + kCtlBytes) / 4; i += blockDim.x)
        *((LdsU32)(red + 4 * i)) = i == (2 * kTileBytes + kCtlNext) / 4 ? (uint32_t)WAVES : 0u;
    __syncthreads();

    // ---- the last wave of the workgroup only writes results.  Stores count in the same
    //      vector-memory counter as the LDS-direct loads, and a store is acknowledged late while
    //      HBM is saturated with reads; a streaming wave that stored would stall its own pipeline.
    if (wave == WAVES) {
        // [first, last] contributing workgroup of a strip that this range holds only a part of
        auto contributors = [&](uint32_t strip, uint32_t &b_lo, uint32_t &b_hi) {
            const uint32_t lo = max(g0, strip * k_blocks), hi = min(g1, (strip + 1) * k_blocks);
            if (hi - lo == k_blocks) return false;
            b_lo = rs.of(strip * k_blocks), b_hi = rs.of((strip + 1) * k_blocks - 1);
            return true;
        };
        // C address of float4 unit u = q * 64 + lane of a strip: token u / 16, rows 4 (u % 16) .. + 3
        auto c_unit = [&](uint32_t strip, uint32_t q, uint32_t lane) {
            const uint32_t u = q * 64 + lane, m = u >> 4, c = u & 15u;
            return C + (int64_t)m * ldc + (int64_t)strip * 64 + 4 * c;
        };
        // Per-lane addresses are formed where they are used, from a copy of the lane number the
        // compiler cannot see through: hoisted out of the task loop they would all stay in
        // registers for the whole loop, beside the tile itself.
        auto opaque_lane = [&]() {
            uint32_t l = lane;
            asm volatile("" : "+v"(l));
            return l;
        };
        for (uint32_t j = 0; j < n_tasks; ++j) {
            const uint32_t strip = task_strip(j), par = j & 1u, tile = red + par * kTileBytes;
            const uint32_t lo = max(g0, strip * k_blocks), hi = min(g1, (strip + 1) * k_blocks);
            while (uniform(lds_poll(ctl + kCtlDone + 4 * par)) != hi - lo) __builtin_amdgcn_s_sleep(4);
            lds_fence();
            f32x4 v[kUnits / 64];
            const uint32_t lane_a = opaque_lane();
#pragma unroll
            for (uint32_t q = 0; q < kUnits / 64; ++q) {
                const uint32_t u = q * 64 + lane_a, m = u >> 4, c = u & 15u;
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
            uint32_t b_lo = 0, b_hi = 0;
            const bool shared = contributors(strip, b_lo, b_hi);
            if (shared && ws.mode == kSumCleared) {
                // the host's clear kernel zeroed the strip's columns before this launch
                const uint32_t lane_b = opaque_lane();
#pragma unroll
                for (uint32_t q = 0; q < kUnits / 64; ++q)
                    if ((int)((q * 64 + lane_b) >> 4) < M)
#pragma unroll
                        for (int i = 0; i < 4; ++i) unsafeAtomicAdd(c_unit(strip, q, lane_b) + i, v[q][i]);
                continue;
            }
            if (shared) {
                // kSumParked.  Every contributor parks its partial tile in its slot of the scratch
                // buffer, counts itself in and, without waiting for either, reads the other
                // contributors' slots; whoever counted last adds the tiles up and stores the strip.
                // A slot word is its own "arrived" flag: slots are all zero bits between launches, a
                // parked +0.0 is written as -0.0 (which adds the same), and the last contributor
                // reads a slot until none of its words is zero, then zeroes it again.  So nothing
                // orders the tile stores against the counter, and the whole exchange is one round
                // trip to memory when the others arrived earlier.
                // The slots are accessed through a buffer descriptor over the slot area: 16-byte
                // loads and stores that the compiler issues and waits for itself, that carry the
                // sc1 bit like the agent-scope atomics on the counter (coherent between the L2s of
                // the chip's dies without cache-wide write-backs or invalidations), and that the
                // hardware checks against the size of the area (an out-of-range read returns zero,
                // an out-of-range write is dropped).  "Volatile": the polling reads must be repeated.
                constexpr int kCoherent = 16 | (int)0x80000000u; // sc1 | volatile (compiler-level)
                // kBatch = slots read at a time: what the wave's registers hold beside its own tile
                // (from eight streaming waves on, a wave has 168 registers)
                constexpr int kBatch = MT == 4 || (MT == 2 && WAVES > 7) ? 1 : 3;
                constexpr uint32_t Q = kUnits / 64;
                const uint32_t self = range_id, voff = opaque_lane() * 16;
                const __amdgpu_buffer_rsrc_t slots = __builtin_amdgcn_make_buffer_rsrc(ws.tiles, 0, (int)ws.tiles_bytes, 0x00020000);
                // byte offset of the slot of workgroup b for this strip: slot 0 of a workgroup holds
                // the strip its range starts in, slot 1 the one it ends in
                auto slot_of = [&](uint32_t b) {
                    const uint32_t first = rs.begin(b) >= strip * k_blocks ? 0u : 1u;
                    return uniform((2 * b + first) * kTileBytes);
                };
                const uint32_t mine = slot_of(self);
#pragma unroll
                for (uint32_t q = 0; q < Q; ++q) {
                    u32x4 w = __builtin_bit_cast(u32x4, v[q]);
                    w.x = w.x ? w.x : 0x80000000u, w.y = w.y ? w.y : 0x80000000u;
                    w.z = w.z ? w.z : 0x80000000u, w.w = w.w ? w.w : 0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b128(w, slots, voff + q * 1024, mine, kCoherent);
                }
                uint32_t old = 0;
                if (lane == 0) old = __hip_atomic_fetch_add(ws.count + b_lo, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const u32x4 zero4 = {0u, 0u, 0u, 0u};
                bool last = false;
                for (uint32_t b = b_lo; b <= b_hi;) {
                    // the next kBatch contributors other than this workgroup
                    uint32_t src[kBatch];
                    uint32_t nb = 0; // slots in this batch (wave-uniform)
#pragma unroll
                    for (int i = 0; i < kBatch; ++i) {
                        if (b == self) ++b;
                        src[i] = slot_of(b <= b_hi ? b : self);
                        if (b <= b_hi) ++b, ++nb;
                    }
                    if (nb == 0) break;
                    u32x4 t[kBatch][Q];
                    // A parked tile arrives within a round trip of its owner's count.  The bound only
                    // matters when the scratch contract was broken (a buffer that was not zero-filled
                    // once, or calls overlapping on it): then this gives up and the strip is wrong.
                    for (uint32_t polls = 0;; ++polls) {
#pragma unroll
                        for (int i = 0; i < kBatch; ++i)
                            if ((uint32_t)i < nb)
#pragma unroll
                                for (uint32_t q = 0; q < Q; ++q)
                                    t[i][q] = __builtin_amdgcn_raw_buffer_load_b128(slots, voff + q * 1024, src[i], kCoherent);
                        if (!last) { // first batch: read before this workgroup knows whether it is the last one
                            if (uniform(old) != b_hi - b_lo) break; // somebody else will finish the strip
                            last = true;
                        }
                        bool missing = false;
#pragma unroll
                        for (int i = 0; i < kBatch; ++i)
                            if ((uint32_t)i < nb)
#pragma unroll
                                for (uint32_t q = 0; q < Q; ++q)
                                    missing |= t[i][q].x == 0u || t[i][q].y == 0u || t[i][q].z == 0u || t[i][q].w == 0u;
                        if (__builtin_amdgcn_ballot_w64(missing) == 0 || polls == (1u << 15)) break;
                        __builtin_amdgcn_s_sleep(8);
                    }
                    if (!last) break;
#pragma unroll
                    for (int i = 0; i < kBatch; ++i)
                        if ((uint32_t)i < nb)
#pragma unroll
                            for (uint32_t q = 0; q < Q; ++q) {
                                v[q] += __builtin_bit_cast(f32x4, t[i][q]);
                                // (same address as the load above, same wave: stays behind it)
                                __builtin_amdgcn_raw_buffer_store_b128(zero4, slots, voff + q * 1024, src[i], kCoherent);
                            }
                }
                if (!last) continue;
                // this workgroup's own slot and the counter go back to zero as well (the same
                // addresses as the stores above, from the same wave: they stay in that order)
#pragma unroll
                for (uint32_t q = 0; q < Q; ++q) __builtin_amdgcn_raw_buffer_store_b128(zero4, slots, voff + q * 1024, mine, kCoherent);
                if (lane == 0) __hip_atomic_store(ws.count + b_lo, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const uint32_t lane_c = opaque_lane();
            if (ws.out_bf16) { // the same unit as four BF16: 8 bytes at the same element offset
                uint16_t *C16 = reinterpret_cast<uint16_t *>(C);
#pragma unroll
                for (uint32_t q = 0; q < kUnits / 64; ++q) {
                    const uint32_t u = q * 64 + lane_c, m = u >> 4, c = u & 15u;
                    const u32x2 packed = {bf16_rne(v[q].x) | (bf16_rne(v[q].y) << 16), bf16_rne(v[q].z) | (bf16_rne(v[q].w) << 16)};
                    if ((int)m < M) *reinterpret_cast<u32x2 *>(C16 + (int64_t)m * ldc + (int64_t)strip * 64 + 4 * c) = packed;
                }
                continue;
            }
#pragma unroll
            for (uint32_t q = 0; q < kUnits / 64; ++q)
                if ((int)((q * 64 + lane_c) >> 4) < M) *reinterpret_cast<f32x4 *>(c_unit(strip, q, lane_c)) = v[q];
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
    // Adds the partial sums of n BlockTiles of task j into the task's LDS tile.  D layout of the
    // 16x16 MFMA: a lane holds token lane % 16 and rows 4 * (lane / 16) .. + 3 of the 16-row
    // block, i.e. one float4 unit.
    auto flush = [&](uint32_t j, uint32_t n) {
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
        // the tile addresses are formed here, from a copy of the lane number the compiler cannot
        // see through: hoisted out of the tile loop they would hold 4 MT + 1 registers for good
        uint32_t l = lane;
        asm volatile("" : "+v"(l));
        const uint32_t m_lane = l & 15u, kgrp = l >> 4;
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
    };

    take_begin();
    take_lookup();
    clear_acc();
    uint32_t acc_j = s_j[0], acc_n = 0;

    // Activation fragments (B operands) of the tile about to be decoded: requested at the top
    // of its step, before the LDS-direct loads of the next tile, and awaited right before the
    // first MFMA, so the L2 round trip is covered by the staging and indexing in between.  The
    // compiler cannot count the LDS-direct loads, so it cannot place that wait: the loads are
    // issued by hand and awaited with vmcnt(S::kLoads), the number of vector-memory
    // instructions every step issues after them.  The fragment registers are operands of the
    // wait, so nothing that uses them can move above it.
    auto request_fragments = [&](uint32_t kb, u32x4 (&f)[2][MT]) {
        const uint16_t *src = A + (size_t)kb * 64;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < MT; ++j)
                asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3" : "=v"(f[kh][j]) : "v"(rowoff[j]), "s"(src), "n"(64 * kh));
    };
    auto fragments_arrived = [&](u32x4 (&f)[2][MT]) {
        static_assert(MT == 1 || MT == 2 || MT == 4, "the wait below names every fragment register");
        if constexpr (MT == 1)
            asm volatile("s_waitcnt vmcnt(%2)" : "+v"(f[0][0]), "+v"(f[1][0]) : "n"(S::kLoads));
        else if constexpr (MT == 2)
            asm volatile("s_waitcnt vmcnt(%4)" : "+v"(f[0][0]), "+v"(f[0][1]), "+v"(f[1][0]), "+v"(f[1][1]) : "n"(S::kLoads));
        else
            asm volatile("s_waitcnt vmcnt(%8)"
                         : "+v"(f[0][0]), "+v"(f[0][1]), "+v"(f[0][2]), "+v"(f[0][3]), "+v"(f[1][0]), "+v"(f[1][1]),
                           "+v"(f[1][2]), "+v"(f[1][3])
                         : "n"(S::kLoads));
    };

    // per-lane addresses shared by both ring positions (the distance between the positions goes
    // into the offset fields of the reads)
    const uint32_t pa0 = plane_address(ring + S::kPlanes, lane);
    const uint32_t l_lane0 = l_lane_of(ring + S::kH, ring + S::kL, lane);

    // One iteration decodes the tile in ring position CUR while position CUR ^ 1 is refilled.
    auto step = [&](auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        wait_dma<0>(); // tile CUR and its L window have landed
        lds_fence();   // all LDS reads of the slot to refill are done; the offsets of the next tile are here
        // the bit-plane bytes of tile CUR's first half are read while the next tile is staged
        HalfIndex h0;
        read_planes<CUR * S::kBytes, 0, false>(pa0, h0);
        u32x4 bfrag[2][MT];
        request_fragments(s_kb[CUR], bfrag);
        take_begin();
        stage(NXT); // (waits for the scalar load of the offsets, issued a tile ago)
        take_lookup();
        if (s_j[CUR] != acc_j) {
            flush(acc_j, acc_n);
            clear_acc();
            acc_j = s_j[CUR], acc_n = 0;
        }
        // L addresses are formed relative to ring position 0 (the distance, three times over,
        // is the constant kLX of the decode), so both positions share their per-lane registers
        const uint32_t slot = ring + CUR * S::kBytes;
        constexpr uint32_t kLX = 3 * CUR * S::kBytes;
        uint32_t h_base = slot + S::kH;
        index_half<true>(h_base, h0);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(s_l[CUR].l), s_l[CUR].big != 0};
        fragments_arrived(bfrag);
        bf16x8 bop[2][MT];
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                bop[kh][j] = __builtin_bit_cast(bf16x8, bfrag[kh][j]);
            }
        decode_block_tile<BASE_M1, CUR * S::kBytes, kLX>(tab, pa0, h0, h_base, l_lane0, fs, [&](int tt, const u32x4 &w) {
            const bf16x8 wop = __builtin_bit_cast(bf16x8, w);
#pragma unroll
            for (int j = 0; j < MT; ++j)
                acc[tt & 3][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, bop[tt >> 2][j], acc[tt & 3][j], 0, 0, 0);
        });
        ++acc_n;
    };
    for (;;) {
        if (!s_valid[0]) break;
        step(std::integral_constant<int, 0>{});
        if (!s_valid[1]) break;
        step(std::integral_constant<int, 1>{});
    }
    if (acc_n) flush(acc_j, acc_n);
    wait_dma<0>();
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
                                                                          float *C, int64_t ldc, int M, int q_active,
                                                                          RangeSplit rs)
{
    static_assert(R >= P && R <= 16, "ready / consumed words are laid out for at most 16 dense slots");
    using S = Slot<LW>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables(smem, bv.base_exp);

    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = dynamic_lds_base();
    const uint32_t ctl = tab + kTableBytes, dense0 = ctl + kPcCtlBytes;
    const uint32_t m_lane = lane & 15u, kgrp = lane >> 4;

    const uint32_t k_blocks = (uint32_t)bv.k_blocks;
    const uint32_t g0 = rs.begin(blockIdx.x), g1 = rs.begin(blockIdx.x + 1);

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
        // time as several tiles' worth of MFMAs.  (With eight consumers a wave has 128 registers,
        // which hold two tiles' fragments of 32 tokens, not four.)
        constexpr int D = MT == 1 ? 4 : MT == 2 ? (Q <= 4 ? 4 : 2) : 1;
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
    TileRef p_t = {kNoTileG, kNoTileOff};
    uint32_t g_taken = 0;
    auto take_begin = [&]() {
        g_taken = 0;
        if (lane == 0)
            g_taken = __hip_atomic_fetch_add((LdsU32)(ctl + kPcNext), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    auto take_lookup = [&]() {
        const uint32_t g = uniform(g_taken);
        p_valid = g < g1;
        p_t = TileRef{kNoTileG, kNoTileOff};
        if (p_valid) {
            p_t.g = g;
            p_t.off = offset_quad(bv, g);
        }
    };
    bool s_valid[2] = {false, false};
    uint32_t s_i[2] = {0u, 0u};
    StagedL s_l[2] = {StagedL{bv.L, 0u}, StagedL{bv.L, 0u}};
    // Issues the Slot::kLoads LDS-direct loads of the pending tile into ring position d.
    auto stage = [&](int d) {
        s_l[d] = stage_tile<LW>(bv, p_t, ring + d * S::kBytes, lane);
        s_valid[d] = p_valid, s_i[d] = p_t.g - g0;
    };

    take_begin();
    take_lookup();
    stage(0);
    take_begin();
    take_lookup();

    auto step = [&](auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1;
        lds_fence(); // all LDS reads of the slot to refill are done
        stage(NXT);
        take_begin();
        wait_dma<S::kLoads>(); // everything older than the tile just staged has landed
        take_lookup();

        const uint32_t slot = ring + CUR * S::kBytes;
        HalfIndex h0;
        const uint32_t pa = plane_address(slot + S::kPlanes, lane);
        read_planes<0, 0, false>(pa, h0);
        uint32_t h_base = slot + S::kH;
        index_half<true>(h_base, h0);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(s_l[CUR].l), s_l[CUR].big != 0};

        // the dense slot must have been read by every consumer before it is overwritten
        const uint32_t i = s_i[CUR], dslot = i % (uint32_t)R, need = (uint32_t)q_active * (i / (uint32_t)R);
        while ((int32_t)(uniform(lds_poll(ctl + kPcConsumed + 4 * dslot)) - need) < 0) __builtin_amdgcn_s_sleep(1);
        const uint32_t out = dense0 + dslot * kDenseBytes + lane * 16;
        decode_block_tile<BASE_M1, 0, 0>(tab, pa, h0, h_base, l_lane_of(slot + S::kH, slot + S::kL, lane), fs,
                                         [&](int tt, const u32x4 &w) {
                                             *((__attribute__((address_space(3))) u32x4 *)(out + tt * 1024)) = w;
                                         });
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
    bv->h_fast = bv->h_units >= 256u ? bv->h_units - 255u : 0u;
    bv->l_fast = bv->l_units >= 512u ? bv->l_units - 511u : 0u;
    bv->base_exp = d->base_exp;
    bv->k_blocks = (int32_t)(d->K / 64);
    bv->strips = (int32_t)(d->N / 64);
    return ZS_OK;
}

// The current device and its number of compute units (queried once per device).
struct DeviceInfo {
    int id, cus;
};
int device_info(DeviceInfo *di)
{
    static std::atomic<int> cus[kMaxDevices];
    if (hipGetDevice(&di->id) != hipSuccess) return ZS_ERR_HIP;
    if (di->id < 0 || di->id >= kMaxDevices) return ZS_ERR_HIP;
    di->cus = cus[di->id].load(std::memory_order_relaxed);
    if (di->cus == 0) {
        if (hipDeviceGetAttribute(&di->cus, hipDeviceAttributeMultiprocessorCount, di->id) != hipSuccess || di->cus < 1)
            return ZS_ERR_HIP;
        cus[di->id].store(di->cus, std::memory_order_relaxed);
    }
    return ZS_OK;
}

// Lets kernel k use `bytes` of dynamic LDS.  The attribute sticks to (kernel, device), so it
// is set once per pair: `done` is the call site's bit set of devices already served.
template <class Kernel>
int allow_big_lds(Kernel k, uint32_t bytes, int device, std::atomic<uint64_t> &done)
{
    if (bytes > kMaxLds) return ZS_ERR_CONFIG;
    if (bytes <= 48 * 1024 || (done.load(std::memory_order_acquire) >> device & 1u)) return ZS_OK;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) !=
        hipSuccess)
        return ZS_ERR_HIP;
    done.fetch_or(1ull << device, std::memory_order_release);
    return ZS_OK;
}

// Compute units assumed by the sizing queries when no device can be asked (they are plain
// host arithmetic and also run on machines without a GPU): those of one MI355X.
constexpr int kDefaultCus = 256;
int cus_or_default()
{
    DeviceInfo di;
    return device_info(&di) == ZS_OK ? di.cus : kDefaultCus;
}

RangeSplit split_ranges(uint32_t total, uint32_t parts) { return RangeSplit{total, parts, total / parts, total % parts}; }

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

// id = index + 1.  The first entry of each (tokens, lw, kernel) triple is the default for it.
// Names: m<tokens per launch>_l<0: 512-byte, 4: 4 KB L window>_w<streaming waves> for
// gemm_stream_kernel, p<tokens per launch>_l<..>_w<producer waves> for gemm_pc_kernel.
const GemmVariant kVariants[] = {
    {"m16_l0_w11", 1, 512, 11, 0}, {"m16_l0_w8", 1, 512, 8, 0},   {"m32_l0_w10", 2, 512, 10, 0},
    {"m32_l0_w7", 2, 512, 7, 0},   {"m16_l4_w7", 1, 4096, 7, 0},  {"m32_l4_w6", 2, 4096, 6, 0},
    {"p64_l0_w7", 1, 512, 7, 4},   {"p128_l0_w7", 2, 512, 7, 4},  {"p256_l0_w7", 2, 512, 7, 8},
    {"p64_l4_w5", 1, 4096, 5, 4},  {"p128_l4_w5", 2, 4096, 5, 4}, {"p256_l4_w5", 2, 4096, 5, 8},
    {"m64_l0_w7", 4, 512, 7, 0},   {"m64_l4_w5", 4, 4096, 5, 0},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

// Workgroups of a ZipGEMM launch: one per CU, fewer when there are fewer BlockTiles.
uint32_t auto_workgroups(uint64_t total, int cus) { return (uint32_t)(total < (uint64_t)cus ? total : (uint64_t)cus); }

// C must start from zero where some workgroup's range begins or ends inside a strip: those
// strips are summed from several workgroups with atomics.
void clear_shared_strips(const BlobView &bv, float *C, int64_t ldc, int M, const RangeSplit &rs, hipStream_t s)
{
    SharedStrips list;
    list.n = 0;
    for (uint32_t b = 1; b < rs.parts; ++b) {
        const uint32_t g = rs.begin(b);
        if (g % (uint32_t)bv.k_blocks == 0) continue;
        const uint32_t strip = g / (uint32_t)bv.k_blocks;
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
// between launches), then two partial tiles of 4096 MT bytes per workgroup.  The header has
// one size for every matrix and configuration, so that a buffer which served one call has
// zero counters for any other.
constexpr uint32_t kMaxSharedCounters = 1024;
constexpr uint32_t kScratchHeaderBytes = kMaxSharedCounters * 4;
size_t shared_sums_bytes(uint32_t wgs, int mt) { return kScratchHeaderBytes + (size_t)2 * wgs * 4096 * (size_t)mt; }

template <int MT, int LW, int WAVES>
int launch_gemm(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, uint32_t wgs,
                int device, void *scratch, bool out_bf16, hipStream_t s)
{
    using S = Slot<LW>;
    constexpr uint32_t lds = StreamLds<MT, LW, WAVES>::kTotal;
    static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
    static_assert(S::kLoads < 64, "vmcnt cannot count that many loads");
    static std::atomic<uint64_t> lds_allowed[2];
    const bool m1 = bv.base_exp < 0;
    auto kern = m1 ? gemm_stream_kernel<MT, LW, WAVES, true> : gemm_stream_kernel<MT, LW, WAVES, false>;
    int rc = allow_big_lds(kern, lds, device, lds_allowed[m1]);
    if (rc != ZS_OK) return rc;
    const RangeSplit rs = split_ranges((uint32_t)bv.strips * (uint32_t)bv.k_blocks, wgs);
    SharedSums ws = {nullptr, nullptr, kSumCleared, out_bf16 ? 1u : 0u, 0u};
    if (out_bf16 && !scratch) return ZS_ERR_SIZE; // partial sums of BF16 output cannot be added on C
    if (scratch) {
        ws.count = static_cast<uint32_t *>(scratch);
        ws.tiles = reinterpret_cast<float *>(static_cast<uint8_t *>(scratch) + kScratchHeaderBytes);
        ws.tiles_bytes = (uint32_t)(shared_sums_bytes(wgs, MT) - kScratchHeaderBytes);
        ws.mode = kSumParked;
    } else {
        clear_shared_strips(bv, C, ldc, M, rs, s);
    }
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(64 * (WAVES + 1)), lds, s, bv, A, lda, C, ldc, M, ws, rs);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

template <int MT, int LW, int P, int R, int Q>
int launch_pc(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, uint32_t wgs,
              int device, hipStream_t s)
{
    using S = Slot<LW>;
    constexpr uint32_t lds = kTableBytes + kPcCtlBytes + R * kDenseBytes + P * 2 * S::kBytes;
    static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
    static_assert(S::kLoads < 64, "vmcnt cannot count that many loads");
    static std::atomic<uint64_t> lds_allowed[2];
    const bool m1 = bv.base_exp < 0;
    auto kern = m1 ? gemm_pc_kernel<MT, LW, P, R, Q, true> : gemm_pc_kernel<MT, LW, P, R, Q, false>;
    int rc = allow_big_lds(kern, lds, device, lds_allowed[m1]);
    if (rc != ZS_OK) return rc;
    const RangeSplit rs = split_ranges((uint32_t)bv.strips * (uint32_t)bv.k_blocks, wgs);
    clear_shared_strips(bv, C, ldc, M, rs, s);
    const int q_active = ((M + 15) / 16 + MT - 1) / MT; // consumers with at least one token
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(64 * (P + Q)), lds, s, bv, A, lda, C, ldc, M, q_active, rs);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

int variant_for(const zs_desc *d, int64_t M, int cus)
{
    // up to 64 tokens every wave decodes and multiplies for itself; beyond, the decode is shared
    const int lw = pick_l_window(d);
    const int tokens = M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : M <= 128 ? 128 : 256;
    const bool shared_decode = tokens > 64;
    // Waves take BlockTiles one at a time, so a workgroup's last round is rarely full.  With few
    // tiles per workgroup fewer waves (faster each, fuller rounds) win: measured on the 8B
    // shapes, 16 tokens: eight beat eleven up to 64 tiles per workgroup; 32 tokens: seven beat
    // ten below 56.
    const int64_t tiles_per_wg = (d->N / 64) * (d->K / 64) / cus;
    int waves = 0;
    if (lw == 512 && tokens == 16 && tiles_per_wg <= 64) waves = 8;
    if (lw == 512 && tokens == 32 && tiles_per_wg < 56) waves = 7;
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
    DeviceInfo di;
    if ((rc = device_info(&di)) != ZS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    static std::atomic<uint64_t> lds_allowed[4];
    auto launch = [&](auto kern, uint32_t lds, int waves, int site) {
        int r = allow_big_lds(kern, lds, di.id, lds_allowed[site]);
        if (r != ZS_OK) return r;
        int64_t wgs = (n_bt + waves - 1) / waves;
        if (wgs > di.cus) wgs = di.cus;
        hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(64 * waves), lds, s, bv, W_out_dev, ldw);
        return hipGetLastError() == hipSuccess ? (int)ZS_OK : (int)ZS_ERR_HIP;
    };
    const bool m1 = d->base_exp < 0;
    if (pick_l_window(d) == 512) {
        // eight waves with three tiles in flight each (measured against 7 x 3 with a 1 KB window,
        // 11 x 2, 10 x 2, 6 x 4 and 5 x 4: 2 to 10 % faster on the 8B shapes)
        constexpr uint32_t lds = kTableBytes + 8 * 3 * Slot<512>::kBytes;
        static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
        return m1 ? launch(decompress_kernel<512, 3, 8, true>, lds, 8, 0)
                  : launch(decompress_kernel<512, 3, 8, false>, lds, 8, 1);
    }
    constexpr uint32_t lds = kTableBytes + 7 * 2 * Slot<4096>::kBytes;
    return m1 ? launch(decompress_kernel<4096, 2, 7, true>, lds, 7, 2)
              : launch(decompress_kernel<4096, 2, 7, false>, lds, 7, 3);
}

extern "C" int zs_compute_units(void) { return cus_or_default(); }

extern "C" int zs_gemm_num_configs(void) { return kNumVariants; }

extern "C" const char *zs_gemm_config_name(int config)
{
    return (config >= 1 && config <= kNumVariants) ? kVariants[config - 1].name : nullptr;
}

extern "C" int zs_gemm_pick_config(const zs_desc *d, int64_t M)
{
    if (!d || M < 1 || zs_desc_validate(d) != ZS_OK) return 0;
    return variant_for(d, M, cus_or_default());
}

namespace {

// What a ZipGEMM call will launch for (d, M, config): the variant, the number of workgroups
// and the scratch bytes its kernel can use (0 for the producer / consumer kernel).
struct GemmPlan {
    int variant;
    uint32_t wgs;
    size_t scratch_bytes;
};
int plan_gemm(const zs_desc *d, int64_t M, int config, int cus, GemmPlan *p)
{
    if (config < 0) return ZS_ERR_CONFIG;
    p->variant = config & 0xFF;
    if (p->variant == 0) p->variant = variant_for(d, M, cus);
    if (p->variant < 1 || p->variant > kNumVariants) return ZS_ERR_CONFIG;
    const GemmVariant &v = kVariants[p->variant - 1];
    const uint64_t total = (uint64_t)(d->N / 64) * (uint64_t)(d->K / 64);
    p->wgs = (uint32_t)(config >> 8); // bits 8 and up of config: number of workgroups (0 = one per CU)
    if (p->wgs == 0) p->wgs = auto_workgroups(total, cus);
    if (p->wgs > total) p->wgs = (uint32_t)total;
    // the producer / consumer kernel sums shared strips with atomics on C and uses no scratch
    p->scratch_bytes = !v.shared_decode() && p->wgs <= kMaxSharedCounters ? shared_sums_bytes(p->wgs, v.mt) : 0;
    return ZS_OK;
}

int gemm_impl(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev, int64_t ldc,
              int64_t M, void *workspace_dev, size_t workspace_bytes, hipStream_t s, int config, const DeviceInfo &di,
              bool out_bf16 = false)
{
    BlobView bv;
    int rc = make_view(d, blob_dev, &bv);
    if (rc != ZS_OK) return rc;
    if (!A_dev || !C_dev) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(A_dev) % 16 || reinterpret_cast<uintptr_t>(C_dev) % 16) return ZS_ERR_ARG;
    if (M < 1 || M > (1 << 20) || lda < d->K || lda % 8 || ldc < d->N || ldc % 4) return ZS_ERR_SHAPE;
    GemmPlan plan;
    // BF16 output exists in the streaming kernel only (at most 64 tokens per launch; more tokens
    // run as 64-token panels) and always goes through the scratch buffer
    if ((rc = plan_gemm(d, out_bf16 && M > 64 ? 64 : M, config, di.cus, &plan)) != ZS_OK) return rc;
    const GemmVariant &v = kVariants[plan.variant - 1];
    if (out_bf16 && v.shared_decode()) return ZS_ERR_CONFIG;
    const uint32_t wgs = plan.wgs;
    // row offsets (token * lda * 2 bytes, token < the launch's width) are 32-bit inside the kernels
    if ((uint64_t)lda * 2u * (uint64_t)v.tokens() >= (1ull << 32)) return ZS_ERR_SHAPE;
    // scratch is optional: without it (or with too little) shared strips go through atomics on C
    void *scratch = nullptr;
    if (workspace_dev && plan.scratch_bytes && reinterpret_cast<uintptr_t>(workspace_dev) % 256 == 0 &&
        workspace_bytes >= plan.scratch_bytes)
        scratch = workspace_dev;
    if (out_bf16 && !scratch) return ZS_ERR_SIZE;
    // tokens beyond the variant's width are handled in successive column panels
    const int width = v.tokens();
    for (int64_t m0 = 0; m0 < M; m0 += width) {
        const int m = (int)((M - m0) < width ? (M - m0) : width);
        const uint16_t *Ap = A_dev + m0 * lda;
        float *Cp = out_bf16 ? reinterpret_cast<float *>(reinterpret_cast<uint16_t *>(C_dev) + m0 * ldc) : C_dev + m0 * ldc;
#define ZS_PC_CASE(ID, MT, LW, P, R, Q) \
    case ID: rc = launch_pc<MT, LW, P, R, Q>(bv, Ap, lda, Cp, ldc, m, wgs, di.id, s); break;
#define ZS_CASE(ID, MT, LW, WAVES) \
    case ID: rc = launch_gemm<MT, LW, WAVES>(bv, Ap, lda, Cp, ldc, m, wgs, di.id, scratch, out_bf16, s); break;
        switch (plan.variant) {
            ZS_CASE(1, 1, 512, 11)
            ZS_CASE(2, 1, 512, 8)
            ZS_CASE(3, 2, 512, 10)
            ZS_CASE(4, 2, 512, 7)
            ZS_CASE(5, 1, 4096, 7)
            ZS_CASE(6, 2, 4096, 6)
            ZS_PC_CASE(7, 1, 512, 7, 7, 4)
            ZS_PC_CASE(8, 2, 512, 7, 7, 4)
            ZS_PC_CASE(9, 2, 512, 7, 7, 8)
            ZS_PC_CASE(10, 1, 4096, 5, 5, 4)
            ZS_PC_CASE(11, 2, 4096, 5, 5, 4)
            ZS_PC_CASE(12, 2, 4096, 5, 5, 8)
            ZS_CASE(13, 4, 512, 7)
            ZS_CASE(14, 4, 4096, 5)
        default: rc = ZS_ERR_CONFIG;
        }
#undef ZS_CASE
#undef ZS_PC_CASE
        if (rc != ZS_OK) return rc;
    }
    return ZS_OK;
}

} // namespace

extern "C" size_t zs_gemm_workspace_ex(const zs_desc *d, int64_t M, int config)
{
    if (!d || M < 1 || zs_desc_validate(d) != ZS_OK) return 0;
    GemmPlan plan;
    return plan_gemm(d, M, config, cus_or_default(), &plan) == ZS_OK ? plan.scratch_bytes : 0;
}
extern "C" size_t zs_gemm_workspace(const zs_desc *d, int64_t M) { return zs_gemm_workspace_ex(d, M, 0); }

extern "C" int zs_gemm_ex(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                          int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream,
                          int config)
{
    DeviceInfo di;
    int rc = device_info(&di);
    if (rc != ZS_OK) return rc;
    return gemm_impl(d, blob_dev, A_dev, lda, C_dev, ldc, M, workspace_dev, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream), config, di);
}

extern "C" int zs_gemm_bf16(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, uint16_t *C_dev,
                            int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    DeviceInfo di;
    int rc = device_info(&di);
    if (rc != ZS_OK) return rc;
    return gemm_impl(d, blob_dev, A_dev, lda, reinterpret_cast<float *>(C_dev), ldc, M, workspace_dev, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream), 0, di, true);
}

extern "C" int zs_gemm(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                       int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    return zs_gemm_ex(d, blob_dev, A_dev, lda, C_dev, ldc, M, workspace_dev, workspace_bytes, hip_stream, 0);
}

// ---- ZipGEMM for callers that cannot allocate ----------------------------------------------
// The scratch buffer of gemm_stream_kernel (strip counters + two partial tiles per workgroup)
// lives in a file-scope device array instead of caller memory.  Sized for the widest variant
// (64 tokens) at kStaticWorkgroups workgroups; every GPU the library runs on holds its own copy
// until the process ends.
namespace {
constexpr uint32_t kStaticWorkgroups = 256;
constexpr size_t kStaticScratchBytes = kScratchHeaderBytes + (size_t)2 * kStaticWorkgroups * 4096 * 4;
}
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {

__global__ void zero_units_kernel(u32x4 *p, uint32_t n) // n 16-byte units
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = u32x4{0u, 0u, 0u, 0u};
}

// Device address of `scratch` on the current device (the array's name is only a host-side
// handle): looked up once per device and kept.
int static_scratch(int device, void **out)
{
    static std::atomic<void *> ptr[kMaxDevices];
    void *p = ptr[device].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZS_ERR_HIP;
        ptr[device].store(p, std::memory_order_release);
    }
    *out = p;
    return ZS_OK;
}
} // namespace

extern "C" int zs_gemm_noalloc(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
                               float *C_dev, int64_t ldc, int64_t M, void *hip_stream)
{
    if (!d || M < 1) return d ? ZS_ERR_SHAPE : ZS_ERR_ARG;
    int rc = zs_desc_validate(d);
    if (rc != ZS_OK) return rc;
    DeviceInfo di;
    if ((rc = device_info(&di)) != ZS_OK) return rc;
    GemmPlan plan;
    if ((rc = plan_gemm(d, M, 0, di.cus, &plan)) != ZS_OK) return rc;
    if (plan.scratch_bytes > kStaticScratchBytes) return ZS_ERR_SIZE; // more workgroups than the array was sized for
    void *ptr = nullptr;
    if ((rc = static_scratch(di.id, &ptr)) != ZS_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (plan.scratch_bytes) {
        // The array keeps whatever the last call left.  Counters and slots must start at zero;
        // a completed call leaves them so, one that overlapped with another may not, so the
        // part this call uses is cleared every time.  A fill kernel, not a memset: callers may
        // be capturing.
        const uint32_t units = (uint32_t)(plan.scratch_bytes / 16);
        hipLaunchKernelGGL(zero_units_kernel, dim3((units + 255) / 256), dim3(256), 0, s, static_cast<u32x4 *>(ptr), units);
        if (hipGetLastError() != hipSuccess) return ZS_ERR_HIP;
    }
    return gemm_impl(d, blob_dev, A_dev, lda, C_dev, ldc, M, ptr, kStaticScratchBytes, s, 0, di);
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
