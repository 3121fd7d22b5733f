// Device-side building blocks shared by the decompression kernel and ZipGEMM (gfx950,
// wave64).  One wave decodes one TensorCoreTile (16 x 32 weights) at a time: lane l owns
// row l % 8 of FragTile l / 8, i.e. one byte of each bit-plane and eight consecutive
// weights along K -- exactly the four operand VGPRs the lane feeds to
// v_mfma_f32_16x16x32_bf16.  The steps follow Algorithm 2 of the ZipServ paper:
//   spatial indicator  m = b1 | b2 | b3                       (one byte per lane)
//   dynamic addressing popcount of m + a wave-wide prefix sum (DPP row_shr / row_bcast)
//   implicit lookup    exponent = base_exp + code             (byte-parallel add)
//   repacking          two BF16 per 32-bit operand register
#ifndef ZS_DEVICE_H
#define ZS_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

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
    int32_t base_exp;
    int32_t k_blocks; // K / 64
    int32_t strips;   // N / 64
};

// ---- LDS layout -------------------------------------------------------------------
// Tables (per workgroup, built once):
//   SEL   256 x 16 B  H-byte selectors of v_perm_b32 for the four operand registers,
//                     indexed by the indicator byte m
//   EXP   3 x 256 x 8 B  plane byte -> its eight bits spread to bytes, weighted 1, 2, 4;
//                     table 1 also carries base_exp, so E = T1[b1] + T2[b2] + T3[b3]
// Slot (per wave): one BlockTile: 1536 B of bit-planes, then its H segment, then its L
// segment, then slack for the aligned over-read of the H gather.
constexpr uint32_t kSelBytes = 256 * 16;
constexpr uint32_t kExpBytes = 3 * 256 * 8;
constexpr uint32_t kTableBytes = kSelBytes + kExpBytes;
constexpr uint32_t kPayloadMax = 8224; // H + L of one BlockTile, both padded to 16
constexpr uint32_t kSlotBytes = 9792;  // 1536 + 8224 + 16 slack, rounded to 64

// Element order inside the four operand registers of a lane.
//   kNatural : (0,1) (2,3) (4,5) (6,7)   -- for storing rows of W
//   kMfma    : (0,2) (1,3) (4,6) (5,7)   -- lets one shift place two exponents at once;
//              the activation operand is permuted the same way, so the MFMA sum is unchanged
enum Order { kNatural = 0, kMfma = 1 };

template <Order ORD>
__device__ __forceinline__ constexpr int elem_of(int reg, int half)
{
    return ORD == kNatural ? 2 * reg + half : 4 * (reg >> 1) + (reg & 1) + 2 * half;
}

__device__ __forceinline__ uint32_t lds_u8(const uint8_t *smem, uint32_t off) { return smem[off]; }
__device__ __forceinline__ uint32_t lds_u16(const uint8_t *smem, uint32_t off)
{
    return *reinterpret_cast<const uint16_t *>(smem + off);
}
__device__ __forceinline__ uint32_t lds_u32(const uint8_t *smem, uint32_t off)
{
    return *reinterpret_cast<const uint32_t *>(smem + off);
}

// Builds the SEL and EXP tables; all threads of the workgroup take part, caller syncs.
template <Order ORD>
__device__ inline void build_tables(uint8_t *tab, int32_t base_exp)
{
    // base_exp = -1 (window starts at exponent 0) is folded in later, see decode_tt
    const uint32_t base = base_exp < 0 ? 0u : (uint32_t)base_exp;
    for (uint32_t m = threadIdx.x; m < 256; m += blockDim.x) {
        uint32_t sel[4];
        for (int reg = 0; reg < 4; ++reg) {
            uint32_t s = 0;
            for (int half = 0; half < 2; ++half) {
                const int e = elem_of<ORD>(reg, half);
                // index of element e among the in-window elements of the row (Algorithm 2)
                const uint32_t idx = __builtin_popcount(m & ((1u << e) - 1u));
                const uint32_t byte = ((m >> e) & 1u) ? idx : 0x0Cu; // 0x0C selects constant 0
                s |= (byte | (byte << 8)) << (16 * half);
            }
            sel[reg] = s;
        }
        *reinterpret_cast<u32x4 *>(tab + 16 * m) = u32x4{sel[0], sel[1], sel[2], sel[3]};
        for (uint32_t plane = 0; plane < 3; ++plane) {
            uint32_t lo = 0, hi = 0;
            for (int i = 0; i < 4; ++i) {
                lo |= ((((m >> i) & 1u) << plane) + (plane == 0 ? base : 0u)) << (8 * i);
                hi |= ((((m >> (i + 4)) & 1u) << plane) + (plane == 0 ? base : 0u)) << (8 * i);
            }
            *reinterpret_cast<u32x2 *>(tab + kSelBytes + plane * 2048 + 8 * m) = u32x2{lo, hi};
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

// Running read positions inside a staged BlockTile (wave-uniform).
struct Cursor {
    uint32_t h; // LDS byte offset of the next unread H byte
    uint32_t l; // LDS byte offset of the next unread L halfword
};

// Decodes TensorCoreTile `tt` of the BlockTile staged at smem[slot ..]; returns the lane's
// eight BF16 weights in four registers, ordered per ORD.
template <Order ORD>
__device__ __forceinline__ u32x4 decode_tt(const uint8_t *smem, uint32_t tab, uint32_t slot, int tt,
                                           Cursor &cur, uint32_t lane, bool base_is_minus_one)
{
    // -- bit-plane bytes of this lane's row, spatial indicator, in-window count
    const uint32_t pb = slot + tt * ZS_TT_BITMAP_BYTES + (lane >> 3) * ZS_FT_BITMAP_BYTES + (lane & 7);
    const uint32_t b1 = lds_u8(smem, pb), b2 = lds_u8(smem, pb + 8), b3 = lds_u8(smem, pb + 16);
    const uint32_t m = b1 | b2 | b3;
    const uint32_t cnt = __builtin_popcount(m);

    // -- dynamic addressing: rows are stored in lane order, so a prefix sum over the wave
    //    gives the start of this row inside H, and (8 * lane - that) its start inside L
    const uint32_t incl = wave_inclusive_scan(cnt);
    const uint32_t excl = incl - cnt;
    const uint32_t total = __builtin_amdgcn_readlane(incl, 63);
    const uint32_t hpos = cur.h + excl;
    uint32_t lpos = cur.l + 2 * (8 * lane - excl);
    cur.h += total;
    cur.l += 2 * (ZS_TT_ELEMS - total);

    // -- gather up to 8 H bytes from an arbitrary byte offset: 3 aligned words + funnel shift
    const uint32_t ha = hpos & ~3u;
    const uint32_t d0 = lds_u32(smem, ha), d1 = lds_u32(smem, ha + 4), d2 = lds_u32(smem, ha + 8);
    const uint32_t h0 = __builtin_amdgcn_alignbyte(d1, d0, hpos & 3u);
    const uint32_t h1 = __builtin_amdgcn_alignbyte(d2, d1, hpos & 3u);

    // -- expand the compacted bytes to element positions, each duplicated into both bytes
    //    of its halfword: bit 15 = sign and bits 6..0 = mantissa are then already in place
    const u32x4 sel = *reinterpret_cast<const u32x4 *>(smem + tab + 16 * m);
    uint32_t r0 = __builtin_amdgcn_perm(h1, h0, sel.x);
    uint32_t r1 = __builtin_amdgcn_perm(h1, h0, sel.y);
    uint32_t r2 = __builtin_amdgcn_perm(h1, h0, sel.z);
    uint32_t r3 = __builtin_amdgcn_perm(h1, h0, sel.w);

    // -- implicit lookup, eight exponents at once: E = base_exp + code, one byte each
    const u32x2 t1 = *reinterpret_cast<const u32x2 *>(smem + tab + kSelBytes + 8 * b1);
    const u32x2 t2 = *reinterpret_cast<const u32x2 *>(smem + tab + kSelBytes + 2048 + 8 * b2);
    const u32x2 t3 = *reinterpret_cast<const u32x2 *>(smem + tab + kSelBytes + 4096 + 8 * b3);
    uint32_t e_lo = t1.x + t2.x + t3.x; // elements 0..3
    uint32_t e_hi = t1.y + t2.y + t3.y; // elements 4..7
    if (base_is_minus_one) {
        // code - 1 per byte without borrowing from a neighbour (bytes with code 0 are fallbacks)
        e_lo = ((e_lo | 0x80808080u) - 0x01010101u) & 0x7F7F7F7Fu;
        e_hi = ((e_hi | 0x80808080u) - 0x01010101u) & 0x7F7F7F7Fu;
    }

    // -- exponent field = bits 14..7 of each halfword
    const uint32_t kExpMask = 0x7F807F80u;
    if (ORD == kMfma) {
        // (E << 7) puts elements 0 and 2 of a 4-byte group into place, (E >> 1) elements 1 and 3
        r0 = ((e_lo << 7) & kExpMask) | (r0 & ~kExpMask);
        r1 = ((e_lo >> 1) & kExpMask) | (r1 & ~kExpMask);
        r2 = ((e_hi << 7) & kExpMask) | (r2 & ~kExpMask);
        r3 = ((e_hi >> 1) & kExpMask) | (r3 & ~kExpMask);
    } else {
        const uint32_t x0 = __builtin_amdgcn_perm(0u, e_lo, 0x010C000Cu) >> 1; // [E1,0,E0,0] >> 1
        const uint32_t x1 = __builtin_amdgcn_perm(0u, e_lo, 0x030C020Cu) >> 1;
        const uint32_t x2 = __builtin_amdgcn_perm(0u, e_hi, 0x010C000Cu) >> 1;
        const uint32_t x3 = __builtin_amdgcn_perm(0u, e_hi, 0x030C020Cu) >> 1;
        r0 = (x0 & kExpMask) | (r0 & ~kExpMask);
        r1 = (x1 & kExpMask) | (r1 & ~kExpMask);
        r2 = (x2 & kExpMask) | (r2 & ~kExpMask);
        r3 = (x3 & kExpMask) | (r3 & ~kExpMask);
    }

    // -- fallback path: every zero bit of m takes the next raw BF16 of the L segment
    uint32_t fb = m ^ 0xFFu;
    while (__builtin_amdgcn_ballot_w64(fb != 0) != 0) {
        if (fb != 0) {
            const uint32_t e = __builtin_ctz(fb);
            fb &= fb - 1;
            const uint32_t v = lds_u16(smem, lpos);
            lpos += 2;
            const uint32_t reg = ORD == kNatural ? (e >> 1) : (((e >> 2) << 1) | (e & 1u));
            const uint32_t half = ORD == kNatural ? (e & 1u) : ((e >> 1) & 1u);
            const uint32_t keep = half ? 0x0000FFFFu : 0xFFFF0000u;
            const uint32_t ins = half ? (v << 16) : v;
            r0 = reg == 0 ? ((r0 & keep) | ins) : r0;
            r1 = reg == 1 ? ((r1 & keep) | ins) : r1;
            r2 = reg == 2 ? ((r2 & keep) | ins) : r2;
            r3 = reg == 3 ? ((r3 & keep) | ins) : r3;
        }
    }
    return u32x4{r0, r1, r2, r3};
}

// Copies one BlockTile (bit-planes + H segment + L segment) from the blob into the wave's
// LDS slot with 16-byte loads; returns the cursor of its first H byte / L halfword.
// Sizes are clamped so that neither the blob sections nor the slot can be overrun,
// whatever the offset array holds.
__device__ inline Cursor stage_block_tile(const BlobView &bv, uint32_t bt, uint8_t *smem, uint32_t slot,
                                          uint32_t lane)
{
    const u32x2 o0 = bv.offsets[bt], o1 = bv.offsets[bt + 1];
    const uint32_t h_start = min(o0.x, bv.h_units), l_start = min(o0.y, bv.l_units);
    uint32_t hu = min(min(o1.x, bv.h_units) - h_start, (uint32_t)(ZS_BT_ELEMS / 16));
    if (o1.x < o0.x) hu = 0;
    uint32_t lu = min(min(o1.y, bv.l_units) - l_start, (uint32_t)(kPayloadMax / 16) - hu);
    if (o1.y < o0.y) lu = 0;

    const u32x4 *src_p = reinterpret_cast<const u32x4 *>(bv.bitmaps + (size_t)bt * ZS_BT_BITMAP_BYTES);
    const u32x4 *src_h = reinterpret_cast<const u32x4 *>(bv.H + (size_t)h_start * 16);
    const u32x4 *src_l = reinterpret_cast<const u32x4 *>(bv.L + (size_t)l_start * 16);
    u32x4 *dst_p = reinterpret_cast<u32x4 *>(smem + slot);
    u32x4 *dst_h = dst_p + ZS_BT_BITMAP_BYTES / 16;
    u32x4 *dst_l = dst_h + hu;
    for (uint32_t i = lane; i < ZS_BT_BITMAP_BYTES / 16; i += 64) dst_p[i] = __builtin_nontemporal_load(src_p + i);
    for (uint32_t i = lane; i < hu; i += 64) dst_h[i] = __builtin_nontemporal_load(src_h + i);
    for (uint32_t i = lane; i < lu; i += 64) dst_l[i] = __builtin_nontemporal_load(src_l + i);
    Cursor c;
    c.h = slot + ZS_BT_BITMAP_BYTES;
    c.l = c.h + hu * 16;
    return c;
}

} // namespace zs
#endif
