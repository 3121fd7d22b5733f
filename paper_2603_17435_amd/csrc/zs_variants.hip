// Decompression kernel for the format variants (Algorithm 2 of the ZipServ paper with n = 2, 3
// or 4 bit-planes; Section 4.2, "The Choice of Codeword Length"), with the two extensions of
// zs_variant_encode: windows per BlockTile or per BlockTile row, and a dense H array.
//
// One wave per BlockTile, eight steps of one TensorCoreTile (16 x 32) each.  Lane l holds row
// l % 8 of FragTile l / 8: eight consecutive elements along K, stored with one 16-byte store.
// Its H cursor is the number of in-window elements before it in storage order: the BlockTile's
// running count, plus the counts of the FragTiles before its own in this step (shuffles), plus
// the popcount of its FragTile's mask below its row.  Its L cursor is what is left of its
// position.  With dense H the byte of element p of FragTile f lies at 64 f + p and only the L
// cursor needs the counts.
//
// Every read of the blob goes through a raw buffer descriptor of the blob's size, so the
// hardware drops anything out of range: offsets read from a corrupt blob cannot fault.  A plain
// kernel for measuring the formats against each other; the tuned path is zs_decompress.
#include <hip/hip_runtime.h>

#include "zipserv.h"
#include "zs_format.h"

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct VariantView {
    const void *blob;
    uint32_t total_bytes;
    uint32_t off_planes, off_offsets, off_bases, off_H, off_L;
    uint32_t n_bt, k_blocks;
    int32_t base_mode, dense_h;
};

constexpr int kWavesPerGroup = 4;

template <int NP>
__global__ __launch_bounds__(64 * kWavesPerGroup) void variant_decompress_kernel(VariantView v, uint16_t *out, int64_t ldo)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t bt = blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);
    if (bt >= v.n_bt) return; // whole wave
    const __amdgpu_buffer_rsrc_t blob = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(v.blob), 0, (int)v.total_bytes, 0x00020000);
    auto word = [&](uint32_t at) { return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(blob, at, 0, 0); };
    auto byte = [&](uint32_t at) { return (uint32_t)(uint8_t)__builtin_amdgcn_raw_buffer_load_b8(blob, at, 0, 0); };
    auto half = [&](uint32_t at) { return (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(blob, at, 0, 0); };
    auto dword2 = [&](uint32_t at) {
        const u32x2 w = __builtin_amdgcn_raw_buffer_load_b64(blob, at, 0, 0);
        return (uint64_t)w.x | ((uint64_t)w.y << 32);
    };

    const uint32_t h_seg = v.off_H + 16u * word(v.off_offsets + 8u * bt);      // first H byte of this BlockTile
    const uint32_t l_seg = v.off_L + 16u * word(v.off_offsets + 8u * bt + 4u); // first L byte
    const uint32_t ft = lane >> 3, r = lane & 7u;
    const uint32_t strip = bt / v.k_blocks, kb = bt - strip * v.k_blocks;
    uint32_t high_before = 0; // in-window elements of the TensorCoreTiles already done
    for (uint32_t tt = 0; tt < ZS_TT_PER_BT; ++tt) {
        const uint32_t f = tt * ZS_FT_PER_TT + ft; // FragTile inside the BlockTile, storage order
        const uint32_t row = 16u * (tt & 3u) + 8u * (ft & 1u) + r, col = 32u * (tt >> 2) + 8u * (ft >> 1);
        uint64_t plane[NP], mask = 0;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            plane[i] = dword2(v.off_planes + (bt * ZS_FT_ELEMS + f) * (8u * NP) + 8u * i);
            mask |= plane[i];
        }
        const uint32_t count = (uint32_t)__builtin_popcountll(mask);
        const uint32_t below = (uint32_t)__builtin_popcountll(mask & ((1ull << (8u * r)) - 1ull));
        uint32_t before = 0, step_total = 0; // in-window elements of the FragTiles before this one / of the step
#pragma unroll
        for (uint32_t j = 0; j < ZS_FT_PER_TT; ++j) {
            const uint32_t c = (uint32_t)__shfl((int)count, (int)(8u * j));
            before += j < ft ? c : 0u;
            step_total += c;
        }
        const uint32_t position = 64u * f + 8u * r;         // elements before this lane's first
        const uint32_t hi = high_before + before + below;   // in-window ones among them
        uint32_t li = position - hi;                        // fallbacks among them
        high_before += step_total;

        // the (up to) eight H bytes of this lane, first one in the low byte
        uint64_t hbytes;
        if (v.dense_h) {
            hbytes = dword2(h_seg + position);
        } else {
            const uint32_t at = h_seg + hi, aligned = at & ~3u, shift = 8u * (at & 3u);
            const uint64_t lo = dword2(aligned);
            const uint32_t top = word(aligned + 8u);
            hbytes = shift ? (lo >> shift) | ((uint64_t)top << (64u - shift)) : lo;
        }
        const uint32_t win_lo = byte(v.off_bases + (v.base_mode == ZS_BASE_ROW ? bt * ZS_BT_DIM + row : bt));
        const uint32_t bits = (uint32_t)(mask >> (8u * r)) & 0xFFu;
        uint32_t code_bits[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) code_bits[i] = (uint32_t)(plane[i] >> (8u * r)) & 0xFFu;
        uint32_t value[8];
#pragma unroll
        for (uint32_t e = 0; e < 8; ++e) {
            uint32_t code = 0;
#pragma unroll
            for (int i = 0; i < NP; ++i) code |= ((code_bits[i] >> e) & 1u) << i;
            const uint32_t b = (uint32_t)hbytes & 0xFFu;
            if ((bits >> e) & 1u) {
                value[e] = ((b & 0x80u) << 8) | (((win_lo - 1u + code) & 0xFFu) << 7) | (b & 0x7Fu);
                hbytes >>= 8;
            } else {
                value[e] = half(l_seg + 2u * li);
                ++li;
                if (v.dense_h) hbytes >>= 8;
            }
        }
        const u32x4 packed = {value[0] | (value[1] << 16), value[2] | (value[3] << 16), value[4] | (value[5] << 16),
                              value[6] | (value[7] << 16)};
        *reinterpret_cast<u32x4 *>(out + ((int64_t)strip * ZS_BT_DIM + row) * ldo + (int64_t)kb * ZS_BT_DIM + col) = packed;
    }
}

} // namespace

extern "C" int zs_variant_decompress(const zs_variant_desc *d, const void *blob_dev, uint16_t *W_out_dev, int64_t ldw,
                                     void *hip_stream)
{
    int rc = zs_variant_validate(d);
    if (rc != ZS_OK) return rc;
    if (!blob_dev || !W_out_dev) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(blob_dev) % ZS_SECTION_ALIGN || reinterpret_cast<uintptr_t>(W_out_dev) % 16) return ZS_ERR_ARG;
    if (ldw < d->K || ldw % 8) return ZS_ERR_SHAPE;
    if (d->total_bytes >= (1ull << 32)) return ZS_ERR_SIZE; // the buffer descriptor counts bytes in 32 bits
    const uint64_t n_bt = (uint64_t)(d->N / ZS_BT_DIM) * (uint64_t)(d->K / ZS_BT_DIM);
    VariantView v;
    v.blob = blob_dev;
    v.total_bytes = (uint32_t)d->total_bytes;
    v.off_planes = (uint32_t)d->off_planes;
    v.off_offsets = (uint32_t)d->off_offsets;
    v.off_bases = (uint32_t)d->off_bases;
    v.off_H = (uint32_t)d->off_H;
    v.off_L = (uint32_t)d->off_L;
    v.n_bt = (uint32_t)n_bt;
    v.k_blocks = (uint32_t)(d->K / ZS_BT_DIM);
    v.base_mode = d->base_mode;
    v.dense_h = d->dense_h;
    const dim3 grid((uint32_t)((n_bt + kWavesPerGroup - 1) / kWavesPerGroup)), block(64 * kWavesPerGroup);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    switch (d->n_planes) {
    case 2: hipLaunchKernelGGL(variant_decompress_kernel<2>, grid, block, 0, s, v, W_out_dev, ldw); break;
    case 3: hipLaunchKernelGGL(variant_decompress_kernel<3>, grid, block, 0, s, v, W_out_dev, ldw); break;
    default: hipLaunchKernelGGL(variant_decompress_kernel<4>, grid, block, 0, s, v, W_out_dev, ldw); break;
    }
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}
