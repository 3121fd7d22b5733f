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
//   [5632, +1024*LCH)    first LCH KB of the L segment
//   64 bytes of slack    for the aligned over-read of the byte gathers
// PARK = bytes of the FP32 partial tile ZipGEMM parks in a free slot between two tasks.
template <int LCH, int PARK>
struct Slot {
    static constexpr uint32_t kPlanes = 0, kH = ZS_BT_BITMAP_BYTES, kL = kH + 4096;
    static constexpr uint32_t kUsed = kL + 1024 * LCH + 64;
    static constexpr uint32_t kBytes = kUsed > (uint32_t)PARK ? kUsed : (uint32_t)PARK;
    static constexpr int kLoads = 2 + 4 + LCH; // LDS-direct instructions per BlockTile
};

struct Segments {
    const uint8_t *h, *l;
    uint32_t h_bytes, l_bytes;
};

// Start and size of BlockTile bt's H and L segments, clamped so that no read can leave the
// blob sections or a slot whatever the offset array holds.
__device__ __forceinline__ Segments segments_of(const BlobView &bv, uint32_t bt)
{
    // the offset array is read-only for the whole launch: reading it through the constant
    // address space lets a wave-uniform index use scalar loads, which do not share the
    // vector-memory counter with the LDS-direct loads
    typedef const u32x2 __attribute__((address_space(4))) *ConstPairs;
    const ConstPairs off = (ConstPairs)(uintptr_t)bv.offsets;
    const u32x2 o0 = off[bt], o1 = off[bt + 1];
    const uint32_t h0 = min(o0.x, bv.h_units), l0 = min(o0.y, bv.l_units);
    const uint32_t h1 = min(max(o1.x, h0), bv.h_units), l1 = min(max(o1.y, l0), bv.l_units);
    Segments s;
    s.h = bv.H + (size_t)h0 * 16;
    s.l = bv.L + (size_t)l0 * 16;
    s.h_bytes = min(h1 - h0, (uint32_t)(ZS_BT_ELEMS / 16)) * 16;
    s.l_bytes = min(l1 - l0, (uint32_t)(2 * ZS_BT_ELEMS / 16)) * 16;
    return s;
}

// Issues the Slot::kLoads LDS-direct loads of BlockTile bt (exactly that many instructions,
// also when !valid: then only lane 0 runs, on a dummy address).
template <int LCH>
__device__ __forceinline__ void issue_block_tile(const BlobView &bv, uint32_t bt, bool valid, uint32_t slot_at,
                                                 uint32_t lane)
{
    using S = Slot<LCH, 0>;
    Segments sg = {bv.H, bv.L, 0u, 0u};
    if (valid) sg = segments_of(bv, bt);
    const uint8_t *planes = bv.bitmaps + (size_t)(valid ? bt : 0u) * ZS_BT_BITMAP_BYTES;
    dma_segment<2>(planes, valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane, bv.bitmaps);
    dma_segment<4>(sg.h, sg.h_bytes, slot_at + S::kH, lane, bv.bitmaps);
    dma_segment<LCH>(sg.l, min(sg.l_bytes, 1024u * LCH), slot_at + S::kL, lane, bv.bitmaps);
}

__device__ __forceinline__ uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }

// Workgroup barrier that orders LDS traffic only.  (__syncthreads() would also wait for every
// outstanding vector-memory operation, i.e. drain the LDS-direct loads in flight.)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// --------------------------------------------------------------------------------------
// Standalone decompression: waves take BlockTiles round-robin; 16 bytes (8 weights) per lane
// and TensorCoreTile are stored row-major.
// --------------------------------------------------------------------------------------
template <int LCH, int DEPTH, int WAVES, bool BASE_M1>
__global__ __launch_bounds__(64 * WAVES) void decompress_kernel(BlobView bv, uint16_t *out, int64_t ldw)
{
    using S = Slot<LCH, 0>;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables<kNatural>(smem, bv.base_exp);
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = uniform((uint32_t)(uintptr_t)smem);
    const uint32_t ring = tab + kTableBytes + wave * (DEPTH * S::kBytes);
    const uint32_t n_bt = (uint32_t)bv.strips * (uint32_t)bv.k_blocks;
    const uint32_t first = blockIdx.x * WAVES + wave, stride = gridDim.x * WAVES;
    const uint32_t row_in_tt = ((lane >> 3) & 1u) * 8u + (lane & 7u); // FragTiles run N-fastest
    const uint32_t col_in_tt = (lane >> 4) * 8u;

#pragma unroll
    for (int j = 0; j < DEPTH - 1; ++j) {
        const uint32_t bt = first + j * stride;
        issue_block_tile<LCH>(bv, bt, bt < n_bt, ring + j * S::kBytes, lane);
    }
    uint32_t cur = 0, nxt = DEPTH - 1; // ring positions of the tile being decoded / being issued
    for (uint32_t bt = first; bt < n_bt; bt += stride) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // every LDS read of the slot about to be refilled is done
        const uint32_t ahead = bt + (DEPTH - 1) * stride;
        issue_block_tile<LCH>(bv, ahead, ahead < n_bt, ring + nxt * S::kBytes, lane);
        wait_dma<(DEPTH - 1) * S::kLoads>();

        const uint32_t slot = ring + cur * S::kBytes;
        const Segments sg = segments_of(bv, bt);
        BlockIndex bi;
        index_block_tile(slot + S::kPlanes, slot + S::kH, slot + S::kL, lane, bi);
        const FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(sg.l), sg.l_bytes > 1024u * LCH};
        const uint32_t strip = bt / (uint32_t)bv.k_blocks, kb = bt % (uint32_t)bv.k_blocks;
        uint16_t *dst = out + ((int64_t)strip * 64 + row_in_tt) * ldw + (int64_t)kb * 64 + col_in_tt;
        auto run = [&](auto careful) {
            decode_block_tile<kNatural, BASE_M1, decltype(careful)::value>(tab, bi, fs, [&](int tt, const u32x4 &w) {
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
// Work split (Section 4.3.1, split-K tiling): a task is a run of BlockTiles along K inside
// one 64-row strip, (strip, ks) with ks < k_splits.  Tasks go round-robin to workgroups; the
// WAVES waves of a workgroup cut the task's run into WAVES consecutive sub-runs, decode and
// multiply independently, then park their 64 x (16 MT) partial tiles in LDS, sum them
// cooperatively, and a dedicated writer wave stores the sum to C (k_splits == 1) or adds it
// to a cleared C with FP32 atomics.  A wave streams the BlockTiles of all its sub-runs as one sequence, so the
// LDS-direct loads of the next task are already in flight while a task is being reduced.
// The activation fragments of a 64-wide K slab (already in B-operand lane order, see
// prep_kernel; L2-resident) are loaded straight into registers at the end of the previous tile.
// --------------------------------------------------------------------------------------
struct SubRun {
    uint32_t strip, b0, b1; // BlockTiles b0, b0 + WAVES, b0 + 2 WAVES, ... < b1 of strip
};

__device__ __forceinline__ SubRun sub_run_of(uint32_t task, uint32_t k_splits, uint32_t k_blocks, uint32_t wave,
                                             uint32_t waves)
{
    const uint32_t strip = task / k_splits, ks = task - strip * k_splits;
    const uint32_t kb0 = k_blocks * ks / k_splits, kb1 = k_blocks * (ks + 1) / k_splits;
    (void)waves;
    // the waves of a workgroup take the BlockTiles of the run round-robin, so that together
    // they read one contiguous, advancing window of the blob (DRAM page locality)
    return SubRun{strip, kb0 + wave < kb1 ? kb0 + wave : kb1, kb1};
}

#ifdef ZS_DBG_TIMING
// debug builds only: accumulate s_memtime deltas between marks into zs_t[]
#define ZS_T(i) { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); uint64_t now = __builtin_readcyclecounter(); if (i > 0) zs_t[i] += now - zs_last; else zs_t[5] += 1; zs_last = now; }
#else
#define ZS_T(i)
#endif

template <int MT, int LCH, int DEPTH, int WAVES, bool BASE_M1>
__global__ __launch_bounds__(64 * (WAVES + 1)) void gemm_stream_kernel(BlobView bv, const uint8_t *frag, float *C,
                                                                  int64_t ldc, int M, int k_splits)
{
    static_assert(DEPTH == 2, "the register-resident activation fragments assume one tile of prefetch");
    using S = Slot<LCH, 4096 * MT>;
    // LDS after the tables: the summed output tile (16 MT tokens x 64 rows, FP32, in units of
    // float4 = 4 consecutive rows; unit (m, c) lives at m * 16 + (c ^ (m & 15)) so that the 16
    // tokens of one MFMA result hit 16 different bank groups), then one word per wave that
    // names the ring slot holding its partial tile, then the rings.
    constexpr uint32_t kUnits = 16 * MT * 16, kFinalBytes = 16 * kUnits, kRedBytes = kFinalBytes + 64;
    static_assert(S::kBytes >= kFinalBytes, "a slot must be able to hold a partial tile");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables<kMfma>(smem, bv.base_exp);
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = uniform(threadIdx.x >> 6);
    const uint32_t tab = uniform((uint32_t)(uintptr_t)smem);
    const uint32_t red = tab + kTableBytes;
    const uint32_t ring0 = red + kRedBytes, ring = ring0 + wave * (DEPTH * S::kBytes);
    const uint32_t n_tasks = (uint32_t)bv.strips * (uint32_t)k_splits;
    const uint32_t m_lane = lane & 15u, kgrp = lane >> 4;

    // ---- the last wave of the workgroup only writes results.  Stores count in the same
    //      vector-memory counter as the LDS-direct loads, and a store is acknowledged late while
    //      HBM is saturated with reads; a streaming wave that stored would stall its own pipeline.
    if (wave == WAVES) {
        for (uint32_t task = blockIdx.x; task < n_tasks; task += gridDim.x) {
            lds_barrier(); // partial tiles parked
            lds_barrier(); // summed tile complete
            const uint32_t strip = task / (uint32_t)k_splits;
#pragma unroll
            for (uint32_t u = lane; u < kUnits; u += 64) {
                const uint32_t m = u >> 4, c = u & 15u;
                const f32x4 v = *((const __attribute__((address_space(3))) f32x4 *)(red + 16 * (m * 16 + (c ^ (m & 15u)))));
                if ((int)m < M) {
                    float *dst = C + (int64_t)m * ldc + (int64_t)strip * 64 + 4 * c;
                    if (k_splits == 1) {
                        *reinterpret_cast<f32x4 *>(dst) = v;
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q) unsafeAtomicAdd(dst + q, v[q]);
                    }
                }
            }
        }
        return;
    }

    // ---- the issuing side walks the wave's BlockTile sequence DEPTH - 1 tiles ahead
    uint32_t it_task = blockIdx.x, it_strip = 0, it_kb = 0, it_end = 0;
    if (it_task < n_tasks) {
        const SubRun r = sub_run_of(it_task, k_splits, bv.k_blocks, wave, WAVES);
        it_strip = r.strip, it_kb = r.b0, it_end = r.b1;
    }
    bool p_valid = false;      // the next BlockTile to issue ...
    uint32_t p_bt = 0, p_kb = 0;
    Segments p_sg = {bv.H, bv.L, 0u, 0u}; // ... and its segments, fetched one step early
    auto fetch = [&]() {
        while (it_task < n_tasks && it_kb >= it_end) {
            it_task += gridDim.x;
            if (it_task < n_tasks) {
                const SubRun r = sub_run_of(it_task, k_splits, bv.k_blocks, wave, WAVES);
                it_strip = r.strip, it_kb = r.b0, it_end = r.b1;
            }
        }
        p_valid = it_task < n_tasks;
        p_sg = Segments{bv.H, bv.L, 0u, 0u};
        if (p_valid) {
            p_kb = it_kb;
            it_kb += WAVES;
            p_bt = it_strip * (uint32_t)bv.k_blocks + p_kb;
            p_sg = segments_of(bv, p_bt);
        }
    };
    // what the decoding side needs to know about a staged tile, per ring position (wave-uniform)
    const uint8_t *info_l[DEPTH];
    bool info_big[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) info_l[d] = bv.L, info_big[d] = false;
    // activation fragments of the tile decoded next: loaded by loads the compiler does not
    // track (they must not make it drain the LDS-direct loads); valid after the next wait_dma
    bool n_valid = false;
    uint32_t n_kb = 0;
    u32x4 bfrag[2][MT];
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int j = 0; j < MT; ++j) bfrag[kh][j] = u32x4{0u, 0u, 0u, 0u};
    auto load_bfrag = [&]() {
        if (n_valid) {
            const uint8_t *src = frag + ((size_t)n_kb * (2 * MT)) * 1024 + lane * 16;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(bfrag[kh][j]) : "v"(src + (kh * MT + j) * 1024) : "memory");
        }
    };
    auto issue = [&](uint32_t slot_idx) {
        const uint32_t slot_at = ring + slot_idx * S::kBytes;
        const uint8_t *planes = bv.bitmaps + (size_t)(p_valid ? p_bt : 0u) * ZS_BT_BITMAP_BYTES;
        dma_segment<2>(planes, p_valid ? ZS_BT_BITMAP_BYTES : 0u, slot_at + S::kPlanes, lane, bv.bitmaps);
        dma_segment<4>(p_sg.h, p_sg.h_bytes, slot_at + S::kH, lane, bv.bitmaps);
        dma_segment<LCH>(p_sg.l, min(p_sg.l_bytes, 1024u * LCH), slot_at + S::kL, lane, bv.bitmaps);
        n_valid = p_valid, n_kb = p_kb;
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (slot_idx == (uint32_t)d) info_l[d] = p_sg.l, info_big[d] = p_sg.l_bytes > 1024u * LCH;
    };

#ifdef ZS_DBG_TIMING
    uint64_t zs_t[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, zs_last = 0;
    zs_t[7] = __builtin_readcyclecounter();
#endif
    fetch();
#pragma unroll
    for (int j = 0; j < DEPTH - 1; ++j) {
        issue(j);
        fetch();
    }
    load_bfrag();
#ifdef ZS_DBG_TIMING
    zs_t[8] = __builtin_readcyclecounter();
#endif
    uint32_t cur = 0, nxt = DEPTH - 1;

    for (uint32_t task = blockIdx.x; task < n_tasks; task += gridDim.x) {
        const SubRun sr = sub_run_of(task, k_splits, bv.k_blocks, wave, WAVES);
        f32x4 acc[4][MT];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (uint32_t kb = sr.b0; kb < sr.b1; kb += WAVES) {
            ZS_T(0)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // all LDS reads of the slot to refill are done
            issue(nxt);
            ZS_T(1)
            fetch();
            wait_dma<(DEPTH - 1) * S::kLoads>(); // everything older than the tile just issued has landed
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j) asm volatile("" : "+v"(bfrag[kh][j]));
            ZS_T(2)

            const uint32_t slot = ring + cur * S::kBytes;
#ifdef ZS_DBG_STREAM_ONLY
            acc[0][0][0] += __builtin_bit_cast(float, lds_u32<0>(slot + lane * 4));
            cur = cur + 1 == DEPTH ? 0 : cur + 1;
            nxt = nxt + 1 == DEPTH ? 0 : nxt + 1;
            continue;
#endif
            BlockIndex bi;
            index_block_tile(slot + S::kPlanes, slot + S::kH, slot + S::kL, lane, bi);
            ZS_T(3)
            FallbackSource fs = {slot + S::kL, reinterpret_cast<const uint16_t *>(info_l[0]), info_big[0]};
#pragma unroll
            for (int d = 1; d < DEPTH; ++d)
                if (cur == (uint32_t)d) fs.l_glob = reinterpret_cast<const uint16_t *>(info_l[d]), fs.from_global = info_big[d];
            bf16x8 bop[2][MT];
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j) bop[kh][j] = __builtin_bit_cast(bf16x8, bfrag[kh][j]);
            auto run = [&](auto careful) {
                decode_block_tile<kMfma, BASE_M1, decltype(careful)::value>(tab, bi, fs, [&](int tt, const u32x4 &w) {
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
            load_bfrag(); // for the tile issued at the top of this iteration
            ZS_T(4)
            cur = cur + 1 == DEPTH ? 0 : cur + 1;
            nxt = nxt + 1 == DEPTH ? 0 : nxt + 1;
        }

        // ---- cross-wave reduction.  The ring slot that will be refilled next is free: park the
        //      partial tile there.  D layout of the 16x16 MFMA: a lane holds token lane % 16 and
        //      rows 4 * (lane / 16) .. + 3 of the 16-row block, i.e. one float4 unit.
        typedef __attribute__((address_space(3))) f32x4 *LdsF32x4;
#ifdef ZS_DBG_TIMING
        const uint64_t zs_r0 = __builtin_readcyclecounter();
#endif
        const uint32_t park = ring + nxt * S::kBytes;
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t m = j * 16 + m_lane, c = i * 4 + kgrp;
                *((LdsF32x4)(park + 16 * (m * 16 + (c ^ (m & 15u))))) = acc[i][j];
            }
        if (lane == 0) *((__attribute__((address_space(3))) uint32_t *)(red + kFinalBytes + 4 * wave)) = park;
        lds_barrier();
        // every wave sums a share of the units over all parked tiles
        for (uint32_t u = wave * 64 + lane; u < kUnits; u += 64 * WAVES) {
            f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < WAVES; ++w) {
                const uint32_t at = uniform(lds_u32<0>(red + kFinalBytes + 4 * w));
                sum += *((LdsF32x4)(at + 16 * u));
            }
            *((LdsF32x4)(red + 16 * u)) = sum;
        }
        lds_barrier();
#ifdef ZS_DBG_TIMING
        zs_t[10] += __builtin_readcyclecounter() - zs_r0;
        zs_t[11] += 1;
#endif
    }
    wait_dma<0>();
#ifdef ZS_DBG_TIMING
    if (blockIdx.x == 3 && wave == 1 && lane == 0) {
        uint64_t *o = (uint64_t *)(frag + (1 << 20));
        zs_t[9] = __builtin_readcyclecounter();
        for (int i = 0; i < 12; ++i) o[i] = zs_t[i];
    }
#endif
}

// Prepares one ZipGEMM launch: (1) writes the activations in B-operand fragment order --
// chunk (kb, kh, j) = 64 lanes x 16 bytes, lane l holding the 8 consecutive k of token
// j * 16 + l % 16 that start at kb * 64 + kh * 32 + 8 * (l / 16), reordered to the
// (0,2)(1,3)(4,6)(5,7) element order of the decoded weights, zeros for tokens >= M;
// (2) clears C when split-K partial sums will be accumulated into it.
__global__ void prep_kernel(const uint16_t *A, int64_t lda, int M, int mt, int64_t k_blocks, uint8_t *frag, float *C,
                            int64_t ldc, int64_t N, int zero_c)
{
    const int64_t n_lanes = k_blocks * 2 * mt * 64;
    const int64_t tid = blockIdx.x * (int64_t)blockDim.x + threadIdx.x, nthreads = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = tid; i < n_lanes; i += nthreads) {
        const int lane = (int)(i & 63);
        const int64_t chunk = i >> 6;
        const int j = (int)(chunk % mt), kh = (int)((chunk / mt) & 1);
        const int64_t kb = chunk / (2 * mt);
        const int m = j * 16 + (lane & 15);
        u32x4 a = u32x4{0u, 0u, 0u, 0u};
        if (m < M) a = *reinterpret_cast<const u32x4 *>(A + (int64_t)m * lda + kb * 64 + kh * 32 + (lane >> 4) * 8);
        u32x4 p;
        p.x = __builtin_amdgcn_perm(a.y, a.x, 0x05040100u);
        p.y = __builtin_amdgcn_perm(a.y, a.x, 0x07060302u);
        p.z = __builtin_amdgcn_perm(a.w, a.z, 0x05040100u);
        p.w = __builtin_amdgcn_perm(a.w, a.z, 0x07060302u);
        *reinterpret_cast<u32x4 *>(frag + i * 16) = p;
    }
    if (zero_c) {
        const int64_t n4 = N / 4;
        for (int64_t i = tid; i < n4 * M; i += nthreads) {
            const int64_t m = i / n4, c = i % n4;
            *reinterpret_cast<f32x4 *>(C + m * ldc + c * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
        }
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

// Window of the L segment staged in LDS, in KB: enough for twice the average BlockTile.
int pick_lch(const zs_desc *d)
{
    const uint64_t n_bt = (uint64_t)(d->N / 64) * (uint64_t)(d->K / 64);
    const uint64_t avg = 2 * d->n_fallback / n_bt; // bytes per BlockTile
    const uint64_t want = d->max_l_units * 16ull < 2 * avg ? d->max_l_units * 16ull : 2 * avg;
    return want <= 1024 ? 1 : 4;
}

struct GemmVariant {
    const char *name;
    int mt, lch, depth, waves;
};

// id = index + 1.  The first entry of each (mt, lch) pair is the default for that pair.
const GemmVariant kVariants[] = {
    {"m16_l1_w10", 1, 1, 2, 10}, {"m16_l1_w8", 1, 1, 2, 8},   {"m16_l1_w6", 1, 1, 2, 6},
    {"m32_l1_w8", 2, 1, 2, 8},   {"m32_l1_w6", 2, 1, 2, 6},   {"m64_l1_w4", 4, 1, 2, 4},
    {"m16_l4_w7", 1, 4, 2, 7},   {"m32_l4_w7", 2, 4, 2, 7},   {"m64_l4_w4", 4, 4, 2, 4},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

size_t frag_bytes(int64_t K, int mt) { return (size_t)(K / 32) * mt * 1024; }

template <int MT, int LCH, int DEPTH, int WAVES>
int launch_gemm(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, int64_t N,
                int k_splits, uint8_t *frag, hipStream_t s)
{
    using S = Slot<LCH, 4096 * MT>;
    constexpr uint32_t lds = kTableBytes + 16 * 16 * MT * 16 + 64 + WAVES * DEPTH * S::kBytes;
    static_assert(lds <= kMaxLds, "variant does not fit the 160 KB of LDS");
    static_assert((DEPTH - 1) * S::kLoads < 64, "vmcnt cannot count that many loads");
    const bool m1 = bv.base_exp < 0;
    auto kern = m1 ? gemm_stream_kernel<MT, LCH, DEPTH, WAVES, true> : gemm_stream_kernel<MT, LCH, DEPTH, WAVES, false>;
    int rc = allow_big_lds(kern, lds);
    if (rc != ZS_OK) return rc;
    {
        const int64_t lanes = (int64_t)bv.k_blocks * 2 * MT * 64;
        const int64_t zero = k_splits > 1 ? (int64_t)M * (N / 4) : 0;
        const int64_t work = lanes > zero ? lanes : zero;
        const int blocks = (int)((work + 255) / 256 < 1024 ? (work + 255) / 256 : 1024);
        hipLaunchKernelGGL(prep_kernel, dim3(blocks), dim3(256), 0, s, A, lda, M, MT, (int64_t)bv.k_blocks, frag, C, ldc,
                           N, k_splits > 1 ? 1 : 0);
    }
    const int64_t tasks = (int64_t)bv.strips * k_splits;
    const int64_t wgs = tasks < kNumCus ? tasks : kNumCus;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(64 * (WAVES + 1)), lds, s, bv, (const uint8_t *)frag, C, ldc, M,
                       k_splits);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

int auto_k_splits(const zs_desc *d, int waves)
{
    // tasks = strips * k_splits are dealt to one workgroup per CU in rounds.  Take the fewest
    // splits (they cost atomics) whose last round is at least 85% full, with sub-runs of at
    // least one BlockTile per wave.
    const int64_t strips = d->N / 64, kb = d->K / 64;
    int best = 1;
    double best_eff = 0.0;
    for (int ks = 1; ks <= 64 && kb / ks >= waves; ++ks) {
        const int64_t tasks = strips * ks, rounds = (tasks + kNumCus - 1) / kNumCus;
        const double eff = (double)tasks / (double)(rounds * kNumCus);
        if (eff >= 0.85) return ks;
        if (eff > best_eff) best_eff = eff, best = ks;
    }
    return best;
}

int variant_for(const zs_desc *d, int64_t M)
{
    const int lch = pick_lch(d);
    const int mt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
    for (int i = 0; i < kNumVariants; ++i)
        if (kVariants[i].mt == mt && kVariants[i].lch == lch) return i + 1;
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
    if (pick_lch(d) == 1) {
        constexpr uint32_t lds = kTableBytes + 7 * 3 * Slot<1, 0>::kBytes;
        return m1 ? launch(decompress_kernel<1, 3, 7, true>, lds, 7) : launch(decompress_kernel<1, 3, 7, false>, lds, 7);
    }
    constexpr uint32_t lds = kTableBytes + 7 * 2 * Slot<4, 0>::kBytes;
    return m1 ? launch(decompress_kernel<4, 2, 7, true>, lds, 7) : launch(decompress_kernel<4, 2, 7, false>, lds, 7);
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
    return frag_bytes(d->K, kVariants[variant - 1].mt);
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
    int variant = config & 0xFF, k_splits = config >> 8;
    if (variant == 0) variant = variant_for(d, M);
    if (variant < 1 || variant > kNumVariants) return ZS_ERR_CONFIG;
    const GemmVariant &v = kVariants[variant - 1];
    if (k_splits == 0) k_splits = auto_k_splits(d, v.waves);
    if (k_splits > d->K / 64) k_splits = (int)(d->K / 64);
    if (workspace_bytes < frag_bytes(d->K, v.mt)) return ZS_ERR_SIZE;
    if (!workspace_dev || reinterpret_cast<uintptr_t>(workspace_dev) % 256) return ZS_ERR_ARG;
    uint8_t *frag = static_cast<uint8_t *>(workspace_dev);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // tokens beyond the variant's width are handled in successive column panels
    const int width = 16 * v.mt;
    for (int64_t m0 = 0; m0 < M; m0 += width) {
        const int m = (int)((M - m0) < width ? (M - m0) : width);
        const uint16_t *Ap = A_dev + m0 * lda;
        float *Cp = C_dev + m0 * ldc;
#define ZS_CASE(ID, MT, LCH, DEPTH, WAVES) \
    case ID: rc = launch_gemm<MT, LCH, DEPTH, WAVES>(bv, Ap, lda, Cp, ldc, m, d->N, k_splits, frag, s); break;
        switch (variant) {
            ZS_CASE(1, 1, 1, 2, 10)
            ZS_CASE(2, 1, 1, 2, 8)
            ZS_CASE(3, 1, 1, 2, 6)
            ZS_CASE(4, 2, 1, 2, 8)
            ZS_CASE(5, 2, 1, 2, 6)
            ZS_CASE(6, 4, 1, 2, 4)
            ZS_CASE(7, 1, 4, 2, 7)
            ZS_CASE(8, 2, 4, 2, 7)
            ZS_CASE(9, 4, 4, 2, 4)
        default: rc = ZS_ERR_CONFIG;
        }
#undef ZS_CASE
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
