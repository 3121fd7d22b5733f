// Device-side building blocks shared by the decompression kernel and ZipGEMM (gfx950,
// wave64).  One wave decodes one BlockTile (64 x 64 weights) at a time, TensorCoreTile by
// TensorCoreTile (16 x 32): lane l owns row l % 8 of FragTile l / 8, i.e. one byte of each
// bit-plane and eight consecutive weights along K -- exactly the four operand VGPRs the
// lane feeds to v_mfma_f32_16x16x32_bf16.  The steps follow Algorithm 2 of the ZipServ paper:
//   spatial indicator  m = b1 | b2 | b3                       (one byte per lane)
//   dynamic addressing popcount of m + a wave-wide prefix sum (DPP row_shr / row_bcast)
//   implicit lookup    exponent = base_exp + code             (byte-parallel add)
//   repacking          two BF16 per 32-bit operand register
// The decode of a BlockTile is straight-line code (no branch per element, row or tile), so
// the LDS reads of one TensorCoreTile overlap the arithmetic of its neighbours.
#ifndef ZS_DEVICE_H
#define ZS_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "zs_format.h"

namespace zs {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// What a kernel needs to know about an encoded matrix (filled on the host from zs_desc).
struct BlobView {
    const uint8_t *bitmaps; // 1536 bytes per BlockTile
    const u32x2 *offsets;   // {H start, L start} per BlockTile, 16-byte units, n_bt + 1 entries
    const uint8_t *H;
    const uint8_t *L;
    uint32_t h_units, l_units; // section sizes in 16-byte units (clamps for every read)
    // A segment that starts below these bounds (16-byte units, exclusive) can be read without
    // looking at its length: 4096 bytes of H, 8192 bytes of L stay inside the section.
    uint32_t h_fast, l_fast;
    int32_t base_exp;
    int32_t k_blocks; // K / 64
    int32_t strips;   // N / 64
};

// ---- LDS access by 32-bit address ----------------------------------------------------
// All LDS traffic of the decode goes through plain 32-bit LDS addresses, so that constant
// displacements land in the offset field of the ds_read instructions.
typedef const __attribute__((address_space(3))) uint8_t *LdsU8;
typedef const __attribute__((address_space(3))) uint16_t *LdsU16;
typedef const __attribute__((address_space(3))) uint32_t *LdsU32;
typedef const __attribute__((address_space(3))) u32x2 *LdsU32x2;
typedef const __attribute__((address_space(3))) u32x4 *LdsU32x4;

template <int IMM = 0>
__device__ __forceinline__ uint32_t lds_u8(uint32_t a) { return ((LdsU8)a)[IMM]; }
__device__ __forceinline__ uint32_t lds_u16(uint32_t a) { return *((LdsU16)a); }
template <int IMM = 0>
__device__ __forceinline__ uint32_t lds_u32(uint32_t a) { return ((LdsU32)a)[IMM / 4]; }
// A 32-bit read that is not merged with its neighbour into a two-word read: a pair whose common
// constant offset exceeds the reach of the two-word form (1020 bytes) would cost an address add.
template <int IMM = 0>
__device__ __forceinline__ uint32_t lds_u32_single(uint32_t a)
{
    return ((const volatile __attribute__((address_space(3))) uint32_t *)a)[IMM / 4];
}
template <int IMM = 0>
__device__ __forceinline__ u32x2 lds_u32x2(uint32_t a) { return ((LdsU32x2)a)[IMM / 8]; }
template <int IMM = 0>
__device__ __forceinline__ u32x4 lds_u32x4(uint32_t a) { return ((LdsU32x4)a)[IMM / 16]; }

// ---- LDS tables (per workgroup, built once) ------------------------------------------
//   SEL   256 x 16 B  v_perm_b32 selectors that expand the compacted H bytes of a row to
//                     element positions, indexed by the indicator byte m
//   FSEL  256 x 16 B  v_perm_b32 selectors that drop the first two fallback halfwords of a
//                     row into their element positions, indexed by m
//   EXP   3 x 256 x 8 B  plane byte -> its eight bits spread to bytes, weighted 1, 2, 4;
//                     table 1 also carries base_exp, so E = T1[b1] + T2[b2] + T3[b3]
constexpr uint32_t kSelOff = 0;
constexpr uint32_t kFselOff = 4096;
constexpr uint32_t kExpOff = 8192;
constexpr uint32_t kTableBytes = 8192 + 3 * 2048;

// A lane's eight weights fill four registers in natural order: (0,1) (2,3) (4,5) (6,7), low
// halfword first.  The exponent tables store the bytes of a 4-element group in the order
// e0, e2, e1, e3: then (E << 7) has e0 and e1 in the exponent fields of one register and
// (E >> 1) has e2 and e3 in those of the next, so one shift places two exponents.
__device__ __forceinline__ constexpr int elem_of(int reg, int half) { return 2 * reg + half; }
__device__ __forceinline__ constexpr int exp_byte_elem(int byte) { return byte == 1 ? 2 : byte == 2 ? 1 : byte; }

// Builds the tables at the start of the workgroup's LDS; every thread takes part and the
// caller synchronises.  base_exp = -1 (window starts at exponent 0) is stored as 0 and
// corrected byte-wise in finish_tt.
__device__ inline void build_tables(uint8_t *tab, int32_t base_exp)
{
    const uint32_t base = base_exp < 0 ? 0u : (uint32_t)base_exp;
    for (uint32_t m = threadIdx.x; m < 256; m += blockDim.x) {
        uint32_t sel[4], fsel[4];
        for (int reg = 0; reg < 4; ++reg) {
            uint32_t s = 0, f = 0;
            for (int half = 0; half < 2; ++half) {
                const int e = elem_of(reg, half);
                // index of element e among the in-window elements of the row (Algorithm 2)
                const uint32_t idx_h = __builtin_popcount(m & ((1u << e) - 1u));
                const uint32_t idx_l = (uint32_t)e - idx_h; // ... among the fallbacks
                const bool high = (m >> e) & 1u;
                const uint32_t hb = high ? idx_h : 0x0Cu; // 0x0C selects the constant 0
                s |= (hb | (hb << 8)) << (16 * half);
                // bytes 0..3 = the decoded register, 4..7 = the first two fallback halfwords
                uint32_t lo = 2 * half, hi = 2 * half + 1;
                if (!high && idx_l < 2) {
                    lo = 4 + 2 * idx_l;
                    hi = 5 + 2 * idx_l;
                }
                f |= (lo | (hi << 8)) << (16 * half);
            }
            sel[reg] = s;
            fsel[reg] = f;
        }
        *reinterpret_cast<u32x4 *>(tab + kSelOff + 16 * m) = u32x4{sel[0], sel[1], sel[2], sel[3]};
        *reinterpret_cast<u32x4 *>(tab + kFselOff + 16 * m) = u32x4{fsel[0], fsel[1], fsel[2], fsel[3]};
        for (uint32_t plane = 0; plane < 3; ++plane) {
            uint32_t lo = 0, hi = 0;
            for (int i = 0; i < 4; ++i) {
                const int e = exp_byte_elem(i);
                lo |= ((((m >> e) & 1u) << plane) + (plane == 0 ? base : 0u)) << (8 * i);
                hi |= ((((m >> (e + 4)) & 1u) << plane) + (plane == 0 ? base : 0u)) << (8 * i);
            }
            *reinterpret_cast<u32x2 *>(tab + kExpOff + plane * 2048 + 8 * m) = u32x2{lo, hi};
        }
    }
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x)
{
    x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xf, 0xf, false); // row_shr:1
    x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xf, 0xf, false); // row_shr:2
    x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xf, 0xf, false); // row_shr:4
    x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xf, 0xf, false); // row_shr:8
    x += __builtin_amdgcn_update_dpp(0u, x, 0x142, 0xa, 0xf, false); // row_bcast:15 -> rows 1, 3
    x += __builtin_amdgcn_update_dpp(0u, x, 0x143, 0xc, 0xf, false); // row_bcast:31 -> rows 2, 3
    return x;
}

// A BlockTile is indexed and decoded in two halves of four TensorCoreTiles (0..3 and 4..7): the
// bit-plane bytes and H positions of one half are all a lane keeps at a time, which is what lets
// the 32-token ZipGEMM run three waves per SIMD.
struct HalfIndex {
    uint32_t planes[12]; // [3 i + j] = the lane's byte of plane j + 1 of the half's TensorCoreTile i
    uint32_t hpos[4];    // LDS address of the row's first H byte
    uint32_t min_cnt;    // fewest in-window elements in any of the lane's four rows
};

// A zero-extending byte read from LDS that the compiler does not track: the value is only
// valid after planes_arrived().  (A tracked byte load whose users sit in another basic block
// is kept as an 8-bit value across the blocks and costs one v_and per byte to extend.)
template <int IMM>
__device__ __forceinline__ uint32_t lds_u8_untracked(uint32_t a)
{
    uint32_t v;
    asm volatile("ds_read_u8 %0, %1 offset:%2" : "=v"(v) : "v"(a), "n"(IMM));
    return v;
}

// Per-lane address of the lane's plane bytes inside a BlockTile's bit-planes.
__device__ __forceinline__ uint32_t plane_address(uint32_t planes_at, uint32_t lane)
{
    return planes_at + (lane >> 3) * ZS_FT_BITMAP_BYTES + (lane & 7);
}

// Issues the reads of the lane's bit-plane bytes of half HALF.  The bit-planes lie at the
// address pa was formed from, plus EXTRA: callers that alternate between slots at a constant
// distance pass the first slot's pa and the distance as EXTRA, which lands in the offset field
// of the reads, so that one per-lane address register serves every slot.
// TRACKED = false: nothing is waited for and the compiler does not know the reads are in
// flight, so the caller can put any other work before index_half, which waits for them
// (WAIT = true).  TRACKED = true: ordinary loads, for reads issued in the straight-line code
// of the decode, where the compiler's own wait counts are exact.
template <uint32_t EXTRA, int HALF, bool TRACKED>
__device__ __forceinline__ void read_planes(uint32_t pa, HalfIndex &hi)
{
#define ZS_LOAD_ROW(I)                                                                                   \
    if constexpr (TRACKED) {                                                                             \
        hi.planes[3 * I] = lds_u8<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + EXTRA>(pa);                      \
        hi.planes[3 * I + 1] = lds_u8<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + 8 + EXTRA>(pa);              \
        hi.planes[3 * I + 2] = lds_u8<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + 16 + EXTRA>(pa);             \
    } else {                                                                                             \
        hi.planes[3 * I] = lds_u8_untracked<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + EXTRA>(pa);            \
        hi.planes[3 * I + 1] = lds_u8_untracked<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + 8 + EXTRA>(pa);    \
        hi.planes[3 * I + 2] = lds_u8_untracked<(4 * HALF + I) * ZS_TT_BITMAP_BYTES + 16 + EXTRA>(pa);   \
    }
    ZS_LOAD_ROW(0) ZS_LOAD_ROW(1) ZS_LOAD_ROW(2) ZS_LOAD_ROW(3)
#undef ZS_LOAD_ROW
}

// Makes the plane registers plain 32-bit values the compiler cannot see through.  WAIT = true
// first waits for untracked reads: every plane register is an operand of the wait, so no
// instruction that uses one can be scheduled above it.  (LDS operations complete in order:
// untracked reads in flight can only make the compiler's own waits longer than needed, never
// too short.)
template <bool WAIT>
__device__ __forceinline__ void planes_arrived(HalfIndex &hi)
{
    uint32_t *p = hi.planes;
    if constexpr (WAIT)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(p[0]), "+v"(p[1]), "+v"(p[2]), "+v"(p[3]), "+v"(p[4]), "+v"(p[5]), "+v"(p[6]), "+v"(p[7]),
                       "+v"(p[8]), "+v"(p[9]), "+v"(p[10]), "+v"(p[11]));
    else
        asm volatile(""
                     : "+v"(p[0]), "+v"(p[1]), "+v"(p[2]), "+v"(p[3]), "+v"(p[4]), "+v"(p[5]), "+v"(p[6]), "+v"(p[7]),
                       "+v"(p[8]), "+v"(p[9]), "+v"(p[10]), "+v"(p[11]));
}

// Spatial indicator + dynamic addressing for half a BlockTile.  The in-window counts of three
// TensorCoreTiles share one 32-bit prefix sum (10 bits each: a tile has <= 512), the fourth
// takes one of its own.  h_base: LDS address of the half's first H byte on entry, of the next
// half's on return (wave-uniform).
template <bool WAIT>
__device__ __forceinline__ void index_half(uint32_t &h_base, HalfIndex &hi)
{
    planes_arrived<WAIT>(hi);
    uint32_t cnt[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) cnt[i] = __builtin_popcount(hi.planes[3 * i] | hi.planes[3 * i + 1] | hi.planes[3 * i + 2]);
    hi.min_cnt = min(min(cnt[0], cnt[1]), min(cnt[2], cnt[3]));
    const uint32_t pk[2] = {cnt[0] | (cnt[1] << 10) | (cnt[2] << 20), cnt[3]};
    uint32_t exc[2], tot[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t inc = wave_inclusive_scan(pk[j]);
        exc[j] = inc - pk[j];
        tot[j] = __builtin_amdgcn_readlane(inc, 63);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t excl = (exc[i / 3] >> (10 * (i % 3))) & 0x3FFu;
        const uint32_t total = (tot[i / 3] >> (10 * (i % 3))) & 0x3FFu;
        hi.hpos[i] = h_base + excl;
        h_base += total;
    }
}

// Rows are stored in lane order, a row has 8 elements and TensorCoreTile t starts after 512 t
// elements, so the fallbacks before the lane's row number 512 t + 8 lane - (in-window elements
// before it) and the row's first fallback lies at
//     l_at + 2 (512 t + 8 lane) - 2 (hpos - h_at) = l_lane - 2 hpos + 1024 t + LX
// with the per-lane constant l_lane = 16 lane + l_at + 2 h_at - LX.  LX is a compile-time constant
// of the caller's choice (0, or three times the distance to a reference slot: then l_lane is the
// same for every slot).  load_tt derives the address from hpos in one instruction and leaves
// 1024 t + LX to the offset field of its reads (kLposStep).
constexpr uint32_t kLposStep = 2 * ZS_TT_ELEMS;
__device__ __forceinline__ uint32_t l_lane_of(uint32_t h_at, uint32_t l_at, uint32_t lane) { return 16 * lane + l_at + 2 * h_at; }

// Where the fallbacks of the current BlockTile are read from.
struct FallbackSource {
    uint32_t l_at;          // LDS address of the staged L segment
    const uint16_t *l_glob; // the same segment in global memory
    bool from_global;       // true when the segment did not fit the staged window (wave-uniform)
};

// Overwrites element e of the lane's eight weights with the raw BF16 v.
__device__ __forceinline__ void insert_element(u32x4 &r, uint32_t e, uint32_t v)
{
    const uint32_t reg = e >> 1, sh = (e & 1u) << 4;
    const uint32_t mask = 0xFFFFu << sh, ins = v << sh; // constants stay literals: no register is held for them
    r.x = reg == 0 ? ((r.x & ~mask) | ins) : r.x;
    r.y = reg == 1 ? ((r.y & ~mask) | ins) : r.y;
    r.z = reg == 2 ? ((r.z & ~mask) | ins) : r.z;
    r.w = reg == 3 ? ((r.w & ~mask) | ins) : r.w;
}

// Everything TensorCoreTile t needs from LDS, fetched ahead of the arithmetic so that the
// reads of tile t + 1 are in flight while tile t is assembled.
struct TileLoads {
    uint32_t d0, d1, d2; // 12 bytes around the row's H bytes
    uint32_t l0, l1;     // 8 bytes around the row's first two fallbacks
    u32x4 sel, fsel;     // v_perm selectors for this row's indicator byte
    u32x2 t1, t2, t3;    // exponent tables of the three plane bytes
    uint32_t m;          // the row's indicator byte (1 = in-window element)
    uint32_t hpos;       // LDS address of the row's first H byte
    uint32_t lpos;       // LDS address of the row's first fallback halfword, minus kLposStep * t + LX
};

// The loads are issued in reverse order of first use: LDS returns data in order, so the wait
// for the first value used (the H words) also covers all the others and is the only one.
template <int T, uint32_t LX>
__device__ __forceinline__ TileLoads load_tt(uint32_t tab, const HalfIndex &hi, uint32_t l_lane)
{
    constexpr int i = T % 4;
    TileLoads q;
    const uint32_t b1 = hi.planes[3 * i], b2 = hi.planes[3 * i + 1], b3 = hi.planes[3 * i + 2];
    const uint32_t m = b1 | b2 | b3;
    q.m = m;
    q.hpos = hi.hpos[i];
    const uint32_t ma = (m << 4) + tab;
    q.fsel = lds_u32x4<kFselOff>(ma);
    // l_lane - 2 hpos in one instruction (LDS addresses are far below 2^23)
    asm("v_mad_i32_i24 %0, %1, -2, %2" : "=v"(q.lpos) : "v"(q.hpos), "v"(l_lane));
    const uint32_t la = q.lpos & ~3u;
    if constexpr (kLposStep * T + LX + 4 <= 1020) {
        q.l0 = lds_u32<kLposStep * T + LX>(la);
        q.l1 = lds_u32<kLposStep * T + LX + 4>(la);
    } else {
        q.l0 = lds_u32_single<kLposStep * T + LX>(la);
        q.l1 = lds_u32_single<kLposStep * T + LX + 4>(la);
    }
    q.t1 = lds_u32x2<kExpOff>((b1 << 3) + tab);
    q.t2 = lds_u32x2<kExpOff + 2048>((b2 << 3) + tab);
    q.t3 = lds_u32x2<kExpOff + 4096>((b3 << 3) + tab);
    q.sel = lds_u32x4<kSelOff>(ma);
    // up to 8 H bytes from an arbitrary byte offset: 3 aligned words, funnel-shifted later
    const uint32_t ha = q.hpos & ~3u;
    q.d2 = lds_u32<8>(ha);
    q.d0 = lds_u32<0>(ha);
    q.d1 = lds_u32<4>(ha);
    return q;
}

// Assembles the lane's eight BF16 weights of TensorCoreTile t from its loads.
// CAREFUL = false handles rows with at most two fallbacks (branch-free); CAREFUL = true adds
// a per-lane loop for the third and later fallbacks of a row, and reads every fallback from
// global memory when the L segment did not fit the staged window.
template <bool BASE_M1, bool CAREFUL, uint32_t LX>
__device__ __forceinline__ u32x4 finish_tt(int t, const TileLoads &q, const FallbackSource &fs)
{
    // -- funnel shift (v_alignbyte_b32 uses only the two low bits of its shift operand)
    const uint32_t hpos = q.hpos;
    const uint32_t h0 = __builtin_amdgcn_alignbyte(q.d1, q.d0, hpos);
    const uint32_t h1 = __builtin_amdgcn_alignbyte(q.d2, q.d1, hpos);

    // -- expand the compacted bytes to element positions, each duplicated into both bytes
    //    of its halfword: bit 15 = sign and bits 6..0 = mantissa are then already in place
    u32x4 r;
    r.x = __builtin_amdgcn_perm(h1, h0, q.sel.x);
    r.y = __builtin_amdgcn_perm(h1, h0, q.sel.y);
    r.z = __builtin_amdgcn_perm(h1, h0, q.sel.z);
    r.w = __builtin_amdgcn_perm(h1, h0, q.sel.w);

    // -- implicit lookup, eight exponents at once: E = base_exp + code, one byte each
    uint32_t e_lo = q.t1.x + q.t2.x + q.t3.x; // elements 0..3
    uint32_t e_hi = q.t1.y + q.t2.y + q.t3.y; // elements 4..7
    if (BASE_M1) {
        // code - 1 per byte without borrowing from a neighbour (bytes with code 0 are fallbacks)
        e_lo = ((e_lo | 0x80808080u) - 0x01010101u) & 0x7F7F7F7Fu;
        e_hi = ((e_hi | 0x80808080u) - 0x01010101u) & 0x7F7F7F7Fu;
    }

    // -- exponent field = bits 14..7 of each halfword
    const uint32_t kExpMask = 0x7F807F80u;
    // table bytes are e0, e2, e1, e3: (E << 7) places e0 | e1, (E >> 1) places e2 | e3
    r.x = ((e_lo << 7) & kExpMask) | (r.x & ~kExpMask);
    r.y = ((e_lo >> 1) & kExpMask) | (r.y & ~kExpMask);
    r.z = ((e_hi << 7) & kExpMask) | (r.z & ~kExpMask);
    r.w = ((e_hi >> 1) & kExpMask) | (r.w & ~kExpMask);

    // -- fallback path, common case: the first two raw BF16 of the row, placed with v_perm
    //    (done for every lane: rows without fallbacks have identity selectors)
    const uint32_t lpos = q.lpos;
    const uint32_t lv = __builtin_amdgcn_alignbyte(q.l1, q.l0, lpos);
    r.x = __builtin_amdgcn_perm(lv, r.x, q.fsel.x);
    r.y = __builtin_amdgcn_perm(lv, r.y, q.fsel.y);
    r.z = __builtin_amdgcn_perm(lv, r.z, q.fsel.z);
    r.w = __builtin_amdgcn_perm(lv, r.w, q.fsel.w);

    if (CAREFUL) {
        uint32_t fb = q.m ^ 0xFFu;
        uint32_t pos = lpos + kLposStep * (uint32_t)t + LX;
        if (!fs.from_global) { // the first two are in place already
            fb &= fb - 1;
            fb &= fb - 1;
            pos += 4;
        }
        while (fb != 0) {
            const uint32_t e = __builtin_ctz(fb);
            fb &= fb - 1;
            // Each branch consumes its own load (the empty asm), so that the wait for it sits
            // in the branch.  A wait placed after the join would cover both sources, and the
            // one for global memory also waits for the LDS-direct loads of the next tile.
            uint32_t v;
            if (fs.from_global) {
                v = fs.l_glob[(pos - fs.l_at) >> 1];
                asm volatile("" : "+v"(v));
            } else {
                v = lds_u16(pos);
                asm volatile("" : "+v"(v));
            }
            pos += 2;
            insert_element(r, e, v);
        }
    }
    return r;
}

// Decodes a BlockTile whose first half is indexed (h0; h_base = LDS address where the second
// half's H bytes start), software-pipelined: the LDS reads of TensorCoreTile t + 1 are issued
// before tile t is assembled.  The second half's plane bytes (at pa + EXTRA, see read_planes)
// are read while tile 1 is assembled and indexed before tile 3 is.  sink(t, weights) receives
// each tile's registers.  Each half runs branch-free when none of its rows has more than two
// fallbacks, else in its "careful" variant (also when the L segment did not fit the staged
// window).
template <bool BASE_M1, uint32_t EXTRA, uint32_t LX, class Sink>
__device__ __forceinline__ void decode_block_tile(uint32_t tab, uint32_t pa, const HalfIndex &h0, uint32_t h_base,
                                                  uint32_t l_lane, const FallbackSource &fs, Sink sink)
{
#define ZS_STAGE_BARRIER __builtin_amdgcn_sched_barrier(0)
    HalfIndex h1;
    TileLoads q4;
    auto first = [&](auto careful) {
        constexpr bool C = decltype(careful)::value;
        TileLoads q = load_tt<0, LX>(tab, h0, l_lane);
        TileLoads nq = load_tt<1, LX>(tab, h0, l_lane);
        ZS_STAGE_BARRIER;
        sink(0, finish_tt<BASE_M1, C, LX>(0, q, fs));
        ZS_STAGE_BARRIER;
        q = nq;
        nq = load_tt<2, LX>(tab, h0, l_lane);
        read_planes<EXTRA, 1, true>(pa, h1);
        ZS_STAGE_BARRIER;
        sink(1, finish_tt<BASE_M1, C, LX>(1, q, fs));
        ZS_STAGE_BARRIER;
        q = nq;
        nq = load_tt<3, LX>(tab, h0, l_lane);
        ZS_STAGE_BARRIER;
        sink(2, finish_tt<BASE_M1, C, LX>(2, q, fs));
        ZS_STAGE_BARRIER;
        q = nq;
        index_half<false>(h_base, h1);
        q4 = load_tt<4, LX>(tab, h1, l_lane);
        ZS_STAGE_BARRIER;
        sink(3, finish_tt<BASE_M1, C, LX>(3, q, fs));
        ZS_STAGE_BARRIER;
    };
    if (fs.from_global || __builtin_amdgcn_ballot_w64(h0.min_cnt < 6) != 0)
        first(std::true_type{});
    else
        first(std::false_type{});
    auto second = [&](auto careful) {
        constexpr bool C = decltype(careful)::value;
        TileLoads q = q4;
        TileLoads nq = load_tt<5, LX>(tab, h1, l_lane);
        ZS_STAGE_BARRIER;
        sink(4, finish_tt<BASE_M1, C, LX>(4, q, fs));
        ZS_STAGE_BARRIER;
        q = nq;
        nq = load_tt<6, LX>(tab, h1, l_lane);
        ZS_STAGE_BARRIER;
        sink(5, finish_tt<BASE_M1, C, LX>(5, q, fs));
        ZS_STAGE_BARRIER;
        q = nq;
        nq = load_tt<7, LX>(tab, h1, l_lane);
        ZS_STAGE_BARRIER;
        sink(6, finish_tt<BASE_M1, C, LX>(6, q, fs));
        ZS_STAGE_BARRIER;
        sink(7, finish_tt<BASE_M1, C, LX>(7, nq, fs));
    };
    if (fs.from_global || __builtin_amdgcn_ballot_w64(h1.min_cnt < 6) != 0)
        second(std::true_type{});
    else
        second(std::false_type{});
#undef ZS_STAGE_BARRIER
}

// ---- LDS-direct staging --------------------------------------------------------------
// One global_load_lds_dwordx4 moves 64 x 16 bytes from per-lane global addresses to a
// contiguous 1 KB window of LDS that starts at the wave-uniform address carried in M0.  The
// compiler does not track these loads: completion is awaited with wait_dma<N>().

// Waits until at most N vector-memory operations of this wave are still in flight.  Loads
// complete in issue order, so this guarantees everything issued before the youngest N.
template <int N>
__device__ __forceinline__ void wait_dma()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Copies `bytes` (multiple of 16, at most CHUNKS KB) from gsrc to LDS at lds_at with exactly
// CHUNKS instructions.  Lanes past the end are switched off, except lane 0, which then
// re-reads `dummy` so that every instruction is issued and counted.  LDS positions past
// `bytes` inside the CHUNKS KB window receive garbage.
//
// gsrc, bytes, lds_at and dummy must be wave-uniform and the wave must have all 64 lanes
// active: the lane mask of every instruction is computed on the scalar unit and written to
// EXEC directly (then restored to all ones), the address is the scalar base plus the lane's
// constant offset lane16 = 16 * lane, so issuing costs no vector instruction and no
// vector-to-scalar round trip.
template <int CHUNKS>
__device__ __forceinline__ void dma_segment(const uint8_t *gsrc, uint32_t bytes, uint32_t lds_at, uint32_t lane16,
                                            const uint8_t *dummy)
{
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        const int32_t rem = (int32_t)bytes - c * 1024;
        const uint32_t n = rem <= 0 ? 0u : min((uint32_t)rem >> 4, 64u);
        const uint64_t mask = n >= 64u ? ~0ull : n == 0u ? 1ull : (1ull << n) - 1ull;
        const uint8_t *base = n ? gsrc + c * 1024 : dummy;
        asm volatile("s_mov_b32 m0, %2\n\t"
                     "s_mov_b64 exec, %3\n\t"
                     "global_load_lds_dwordx4 %0, %1\n\t"
                     "s_mov_b64 exec, -1" ::"v"(lane16),
                     "s"(base), "s"(lds_at + c * 1024), "s"(mask)
                     : "memory", "m0");
    }
}

} // namespace zs
#endif
