// Host packer for the format variants (Section 4.2 of the ZipServ paper, "The Choice of Codeword
// Length": codewords of n = 2, 3 or 4 bits; Algorithm 1 with a window of 2^n - 1 exponents),
// plus two extensions the paper does not have: a window per BlockTile or per BlockTile row,
// and a dense H array.  Integer only; the result does not depend on the number of threads.
#include "zipserv.h"
#include "zs_format.h"

#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

namespace {

constexpr uint32_t kVariantVersion = 1;

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

inline bool known_variant(int n_planes, int base_mode, int dense_h)
{
    return n_planes >= 2 && n_planes <= 4 && base_mode >= ZS_BASE_MATRIX && base_mode <= ZS_BASE_ROW &&
           (dense_h == 0 || dense_h == 1);
}

inline uint64_t bases_per_bt(int base_mode) { return base_mode == ZS_BASE_ROW ? ZS_BT_DIM : 1; }

// Start of the run of `width` consecutive exponents with the largest count; the smallest start
// wins a tie (Algorithm 1, phase I).
template <class Count>
int best_window(const Count *hist, int width)
{
    uint64_t sum = 0;
    for (int j = 0; j < width; ++j) sum += hist[j];
    uint64_t best = sum;
    int start = 0;
    for (int s = 1; s + width <= 256; ++s) {
        sum += hist[s + width - 1];
        sum -= hist[s - 1];
        if (sum > best) best = sum, start = s;
    }
    return start;
}

template <class F>
void for_each_strip(int64_t n_strips, int threads, F fn)
{
    const int nt = (int)std::min<int64_t>(std::max(threads, 1), n_strips);
    if (nt <= 1) {
        for (int64_t s = 0; s < n_strips; ++s) fn(s, 0);
        return;
    }
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t)
        pool.emplace_back([=] {
            const int64_t lo = n_strips * t / nt, hi = n_strips * (t + 1) / nt;
            for (int64_t s = lo; s < hi; ++s) fn(s, t);
        });
    for (auto &th : pool) th.join();
}

} // namespace

extern "C" size_t zs_variant_bound(int64_t N, int64_t K, int n_planes, int base_mode, int dense_h)
{
    if (N <= 0 || K <= 0 || N % ZS_BT_DIM || K % ZS_BT_DIM || !known_variant(n_planes, base_mode, dense_h)) return 0;
    const uint64_t n_bt = (uint64_t)(N / ZS_BT_DIM) * (uint64_t)(K / ZS_BT_DIM), elems = (uint64_t)N * (uint64_t)K;
    uint64_t bytes = align_up(n_bt * ZS_FT_ELEMS * 8 * (uint64_t)n_planes, ZS_SECTION_ALIGN);
    bytes += align_up((n_bt + 1) * 8, ZS_SECTION_ALIGN);
    bytes += align_up(n_bt * bases_per_bt(base_mode), ZS_SECTION_ALIGN);
    bytes += align_up(elems + 16 * n_bt, ZS_SECTION_ALIGN);     // H at its worst
    bytes += align_up(2 * elems + 16 * n_bt, ZS_SECTION_ALIGN); // L at its worst
    return (size_t)bytes;
}

extern "C" int zs_variant_validate(const zs_variant_desc *d)
{
    if (!d) return ZS_ERR_ARG;
    if (d->magic != ZS_VARIANT_MAGIC || d->version != kVariantVersion) return ZS_ERR_FORMAT;
    if (!known_variant(d->n_planes, d->base_mode, d->dense_h)) return ZS_ERR_CONFIG;
    if (d->N <= 0 || d->K <= 0 || d->N % ZS_BT_DIM || d->K % ZS_BT_DIM) return ZS_ERR_SHAPE;
    const uint64_t elems = (uint64_t)d->N * (uint64_t)d->K, n_bt = elems / ZS_BT_ELEMS;
    if (d->n_high + d->n_fallback != elems) return ZS_ERR_FORMAT;
    if (d->h_bytes % 16 || d->l_bytes % 16) return ZS_ERR_FORMAT;
    const uint64_t h_elems = d->dense_h ? elems : d->n_high;
    if (d->h_bytes < h_elems || d->h_bytes > h_elems + 15 * n_bt) return ZS_ERR_FORMAT;
    if (d->l_bytes < 2 * d->n_fallback || d->l_bytes > 2 * d->n_fallback + 15 * n_bt) return ZS_ERR_FORMAT;
    const uint64_t offs[5] = {d->off_planes, d->off_offsets, d->off_bases, d->off_H, d->off_L};
    const uint64_t lens[5] = {n_bt * ZS_FT_ELEMS * 8 * (uint64_t)d->n_planes, (n_bt + 1) * 8,
                              n_bt * bases_per_bt(d->base_mode), d->h_bytes, d->l_bytes};
    uint64_t cursor = 0;
    for (int i = 0; i < 5; ++i) {
        if (offs[i] % ZS_SECTION_ALIGN || offs[i] < cursor) return ZS_ERR_FORMAT;
        cursor = offs[i] + lens[i];
    }
    return cursor > d->total_bytes ? ZS_ERR_FORMAT : ZS_OK;
}

extern "C" int zs_variant_encode(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, int n_planes, int base_mode,
                                 int dense_h, void *blob, size_t blob_cap, zs_variant_desc *out, int threads)
{
    if (!W || !blob || !out) return ZS_ERR_ARG;
    if (!known_variant(n_planes, base_mode, dense_h)) return ZS_ERR_CONFIG;
    if (N <= 0 || K <= 0 || N % ZS_BT_DIM || K % ZS_BT_DIM || ldw < K) return ZS_ERR_SHAPE;
    if (blob_cap < zs_variant_bound(N, K, n_planes, base_mode, dense_h)) return ZS_ERR_SIZE;
    if (threads <= 0) threads = (int)std::max(1u, std::thread::hardware_concurrency());

    const int width = (1 << n_planes) - 1;
    const int64_t n_strips = N / ZS_BT_DIM, bts_per_strip = K / ZS_BT_DIM;
    const uint64_t n_bt = (uint64_t)n_strips * (uint64_t)bts_per_strip, per_bt = bases_per_bt(base_mode);
    const uint64_t plane_bytes_bt = (uint64_t)ZS_FT_ELEMS * 8 * (uint64_t)n_planes;
    uint8_t *base = static_cast<uint8_t *>(blob);

    const uint64_t off_planes = 0;
    const uint64_t off_offsets = align_up(n_bt * plane_bytes_bt, ZS_SECTION_ALIGN);
    const uint64_t off_bases = align_up(off_offsets + (n_bt + 1) * 8, ZS_SECTION_ALIGN);
    const uint64_t off_H = align_up(off_bases + n_bt * per_bt, ZS_SECTION_ALIGN);
    std::memset(base + n_bt * plane_bytes_bt, 0, (size_t)(off_offsets - n_bt * plane_bytes_bt));
    std::memset(base + off_offsets + (n_bt + 1) * 8, 0, (size_t)(off_bases - (off_offsets + (n_bt + 1) * 8)));
    std::memset(base + off_bases + n_bt * per_bt, 0, (size_t)(off_H - (off_bases + n_bt * per_bt)));

    // ---- pass 1: windows (Algorithm 1, phase I, per matrix / BlockTile / BlockTile row)
    int matrix_lo = 0;
    if (base_mode == ZS_BASE_MATRIX) {
        std::vector<uint64_t> partial((size_t)threads * 256, 0);
        for_each_strip(n_strips, threads, [&](int64_t strip, int t) {
            uint64_t *h = &partial[(size_t)t * 256];
            for (int64_t n = strip * ZS_BT_DIM; n < (strip + 1) * ZS_BT_DIM; ++n)
                for (int64_t k = 0; k < K; ++k) h[(W[n * ldw + k] >> 7) & 0xFFu]++;
        });
        uint64_t hist[256] = {0};
        for (int t = 0; t < threads; ++t)
            for (int e = 0; e < 256; ++e) hist[e] += partial[(size_t)t * 256 + e];
        matrix_lo = best_window(hist, width);
    }
    uint8_t *bases = base + off_bases;
    // ---- pass 2: per-BlockTile windows and in-window counts
    std::vector<uint32_t> n_high_bt(n_bt);
    for_each_strip(n_strips, threads, [&](int64_t strip, int) {
        for (int64_t kb = 0; kb < bts_per_strip; ++kb) {
            const uint64_t bt = (uint64_t)(strip * bts_per_strip + kb);
            const uint16_t *tile = W + strip * ZS_BT_DIM * ldw + kb * ZS_BT_DIM;
            int tile_lo = matrix_lo;
            if (base_mode == ZS_BASE_TILE) {
                uint32_t hist[256] = {0};
                for (int r = 0; r < ZS_BT_DIM; ++r)
                    for (int k = 0; k < ZS_BT_DIM; ++k) hist[(tile[r * ldw + k] >> 7) & 0xFFu]++;
                tile_lo = best_window(hist, width);
            }
            if (base_mode != ZS_BASE_ROW) bases[bt] = (uint8_t)tile_lo;
            uint32_t c = 0;
            for (int r = 0; r < ZS_BT_DIM; ++r) {
                const uint16_t *row = tile + r * ldw;
                int lo = tile_lo;
                if (base_mode == ZS_BASE_ROW) {
                    uint32_t hist[256] = {0};
                    for (int k = 0; k < ZS_BT_DIM; ++k) hist[(row[k] >> 7) & 0xFFu]++;
                    lo = best_window(hist, width);
                    bases[bt * ZS_BT_DIM + r] = (uint8_t)lo;
                }
                for (int k = 0; k < ZS_BT_DIM; ++k) c += (((row[k] >> 7) & 0xFFu) - (unsigned)lo) < (unsigned)width;
            }
            n_high_bt[bt] = c;
        }
    });

    uint32_t *offsets = reinterpret_cast<uint32_t *>(base + off_offsets);
    uint64_t h_units = 0, l_units = 0, n_high = 0;
    for (uint64_t bt = 0; bt < n_bt; ++bt) {
        offsets[2 * bt + 0] = (uint32_t)h_units;
        offsets[2 * bt + 1] = (uint32_t)l_units;
        const uint32_t nh = n_high_bt[bt], nl = ZS_BT_ELEMS - nh;
        h_units += dense_h ? ZS_BT_ELEMS / 16 : (nh + 15) / 16;
        l_units += (2 * nl + 15) / 16;
        n_high += nh;
    }
    offsets[2 * n_bt + 0] = (uint32_t)h_units;
    offsets[2 * n_bt + 1] = (uint32_t)l_units;
    const uint64_t off_L = align_up(off_H + h_units * 16, ZS_SECTION_ALIGN);
    const uint64_t total = align_up(off_L + l_units * 16, ZS_SECTION_ALIGN);
    if (total > blob_cap) return ZS_ERR_SIZE;
    std::memset(base + off_H + h_units * 16, 0, (size_t)(off_L - (off_H + h_units * 16)));
    std::memset(base + off_L + l_units * 16, 0, (size_t)(total - (off_L + l_units * 16)));

    // ---- pass 3: tile encoding (Algorithm 1, phase II)
    for_each_strip(n_strips, threads, [&](int64_t strip, int) {
        for (int64_t kb = 0; kb < bts_per_strip; ++kb) {
            const uint64_t bt = (uint64_t)(strip * bts_per_strip + kb);
            uint64_t *planes = reinterpret_cast<uint64_t *>(base + off_planes + bt * plane_bytes_bt);
            uint8_t *h = base + off_H + (uint64_t)offsets[2 * bt] * 16;
            uint16_t *l = reinterpret_cast<uint16_t *>(base + off_L + (uint64_t)offsets[2 * bt + 1] * 16);
            uint8_t *h_end = base + off_H + (uint64_t)offsets[2 * bt + 2] * 16;
            uint16_t *l_end = reinterpret_cast<uint16_t *>(base + off_L + (uint64_t)offsets[2 * bt + 3] * 16);
            const uint16_t *tile = W + strip * ZS_BT_DIM * ldw + kb * ZS_BT_DIM;
            for (int tt = 0; tt < ZS_TT_PER_BT; ++tt)
                for (int ft = 0; ft < ZS_FT_PER_TT; ++ft) {
                    const int row0 = 16 * (tt & 3) + 8 * (ft & 1), col0 = 32 * (tt >> 2) + 8 * (ft >> 1);
                    uint64_t plane[4] = {0, 0, 0, 0};
                    for (int r = 0; r < 8; ++r) {
                        const uint16_t *src = tile + (row0 + r) * ldw + col0;
                        const unsigned lo = base_mode == ZS_BASE_ROW ? bases[bt * ZS_BT_DIM + row0 + r] : bases[bt];
                        for (int c = 0; c < 8; ++c) {
                            const uint16_t w = src[c];
                            const unsigned d = ((w >> 7) & 0xFFu) - lo;
                            if (d < (unsigned)width) {
                                const uint64_t code = d + 1;
                                const int p = 8 * r + c;
                                for (int i = 0; i < n_planes; ++i) plane[i] |= ((code >> i) & 1) << p;
                                *h++ = (uint8_t)(((w >> 8) & 0x80u) | (w & 0x7Fu));
                            } else {
                                *l++ = w;
                                if (dense_h) *h++ = 0;
                            }
                        }
                    }
                    for (int i = 0; i < n_planes; ++i) planes[(size_t)n_planes * (tt * ZS_FT_PER_TT + ft) + i] = plane[i];
                }
            while (h < h_end) *h++ = 0;
            while (l < l_end) *l++ = 0;
        }
    });

    std::memset(out, 0, sizeof *out);
    out->magic = ZS_VARIANT_MAGIC;
    out->version = kVariantVersion;
    out->n_planes = n_planes;
    out->base_mode = base_mode;
    out->dense_h = dense_h;
    out->N = N;
    out->K = K;
    out->n_high = n_high;
    out->n_fallback = (uint64_t)N * (uint64_t)K - n_high;
    out->off_planes = off_planes;
    out->off_offsets = off_offsets;
    out->off_bases = off_bases;
    out->off_H = off_H;
    out->off_L = off_L;
    out->h_bytes = h_units * 16;
    out->l_bytes = l_units * 16;
    out->total_bytes = total;
    return ZS_OK;
}
