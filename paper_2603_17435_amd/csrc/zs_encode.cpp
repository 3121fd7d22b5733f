// Host-side TCA-TBE packer (Algorithm 1 and Section 4.2 of the ZipServ paper).
// Three passes over 64-row strips, each split across worker threads:
//   1. exponent histogram                      -> window of 7 consecutive exponents
//   2. per-BlockTile counts of in-window elements -> segment offsets (prefix sum)
//   3. bit-planes, H bytes and L halfwords written at their final place
// Integer only; the result does not depend on the number of threads.
#include "zipserv.h"
#include "zs_format.h"

#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

static_assert(sizeof(zs_desc) == 112, "zs_desc layout is part of the ABI");

namespace {

struct Sections {
    uint64_t off_bitmaps, off_offsets, off_H, off_L;
};

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// Runs fn(strip) for every strip, strips dealt out in contiguous ranges.
template <class F>
void for_each_strip(int64_t n_strips, int threads, F fn)
{
    int nt = (int)std::min<int64_t>(std::max(threads, 1), n_strips);
    if (nt <= 1) {
        for (int64_t s = 0; s < n_strips; ++s) fn(s, 0);
        return;
    }
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t)
        pool.emplace_back([=] {
            int64_t lo = n_strips * t / nt, hi = n_strips * (t + 1) / nt;
            for (int64_t s = lo; s < hi; ++s) fn(s, t);
        });
    for (auto &th : pool) th.join();
}

inline bool in_window(uint16_t w, unsigned win_lo)
{
    unsigned e = (w >> 7) & 0xFFu;
    return e - win_lo < 7u; // unsigned wrap makes this win_lo <= e <= win_lo + 6
}

// First row / first column of FragTile (tt, ft) inside its BlockTile.
inline void fragtile_origin(int tt, int ft, int &row0, int &col0)
{
    row0 = 16 * (tt & 3) + 8 * (ft & 1);
    col0 = 32 * (tt >> 2) + 8 * (ft >> 1);
}

} // namespace

extern "C" size_t zs_encode_bound(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0 || N % ZS_BT_DIM || K % ZS_BT_DIM) return 0;
    uint64_t n_bt = (uint64_t)(N / ZS_BT_DIM) * (uint64_t)(K / ZS_BT_DIM);
    uint64_t elems = (uint64_t)N * (uint64_t)K;
    uint64_t bytes = align_up(n_bt * ZS_BT_BITMAP_BYTES, ZS_SECTION_ALIGN);
    bytes += align_up((n_bt + 1) * 8, ZS_SECTION_ALIGN);
    // any mix of H and L costs at most 2 bytes per element plus 15 bytes of padding per
    // segment; reserve both sections at their individual worst case
    bytes += align_up(elems + 16 * n_bt, ZS_SECTION_ALIGN);
    bytes += align_up(2 * elems + 16 * n_bt, ZS_SECTION_ALIGN);
    return (size_t)bytes;
}

extern "C" int zs_desc_validate(const zs_desc *d)
{
    if (!d) return ZS_ERR_ARG;
    if (d->magic != ZS_MAGIC || d->version != ZS_FORMAT_VERSION || d->tile_cfg != ZS_TILE_CFG_FT8_TT16x32_BT64)
        return ZS_ERR_FORMAT;
    if (d->N <= 0 || d->K <= 0 || d->N % ZS_BT_DIM || d->K % ZS_BT_DIM) return ZS_ERR_SHAPE;
    if (d->base_exp < -1 || d->base_exp > 248) return ZS_ERR_FORMAT;
    uint64_t elems = (uint64_t)d->N * (uint64_t)d->K;
    uint64_t n_bt = elems / ZS_BT_ELEMS;
    if (d->n_high + d->n_fallback != elems) return ZS_ERR_FORMAT;
    if (d->h_bytes % 16 || d->l_bytes % 16) return ZS_ERR_FORMAT;
    if (d->h_bytes < d->n_high || d->h_bytes > d->n_high + 15 * n_bt) return ZS_ERR_FORMAT;
    if (d->l_bytes < 2 * d->n_fallback || d->l_bytes > 2 * d->n_fallback + 15 * n_bt) return ZS_ERR_FORMAT;
    if (d->max_h_units > ZS_BT_ELEMS / 16 || d->max_l_units > 2 * ZS_BT_ELEMS / 16) return ZS_ERR_FORMAT;
    const uint64_t offs[4] = {d->off_bitmaps, d->off_offsets, d->off_H, d->off_L};
    const uint64_t lens[4] = {n_bt * ZS_BT_BITMAP_BYTES, (n_bt + 1) * 8, d->h_bytes, d->l_bytes};
    uint64_t cursor = 0;
    for (int i = 0; i < 4; ++i) {
        if (offs[i] % ZS_SECTION_ALIGN || offs[i] < cursor) return ZS_ERR_FORMAT;
        cursor = offs[i] + lens[i];
    }
    if (cursor > d->total_bytes) return ZS_ERR_FORMAT;
    return ZS_OK;
}

extern "C" int zs_encode(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, void *blob, size_t blob_cap,
                         zs_desc *out, int threads)
{
    if (!W || !blob || !out) return ZS_ERR_ARG;
    if (N <= 0 || K <= 0 || N % ZS_BT_DIM || K % ZS_BT_DIM || ldw < K) return ZS_ERR_SHAPE;
    if (blob_cap < zs_encode_bound(N, K)) return ZS_ERR_SIZE;
    if (threads <= 0) threads = (int)std::max(1u, std::thread::hardware_concurrency());

    const int64_t n_strips = N / ZS_BT_DIM, bts_per_strip = K / ZS_BT_DIM;
    const uint64_t n_bt = (uint64_t)n_strips * (uint64_t)bts_per_strip;

    // ---- pass 1: exponent histogram -> window (Algorithm 1, phase I)
    std::vector<uint64_t> partial((size_t)threads * 256, 0);
    for_each_strip(n_strips, threads, [&](int64_t strip, int t) {
        uint64_t *h = &partial[(size_t)t * 256];
        for (int64_t n = strip * ZS_BT_DIM; n < (strip + 1) * ZS_BT_DIM; ++n) {
            const uint16_t *row = W + n * ldw;
            for (int64_t k = 0; k < K; ++k) h[(row[k] >> 7) & 0xFFu]++;
        }
    });
    uint64_t hist[256] = {0};
    for (int t = 0; t < threads; ++t)
        for (int e = 0; e < 256; ++e) hist[e] += partial[(size_t)t * 256 + e];
    uint64_t window_sum = 0;
    for (int j = 0; j < ZS_WINDOW; ++j) window_sum += hist[j];
    uint64_t best_sum = window_sum;
    int win_lo = 0;
    for (int s = 1; s + ZS_WINDOW <= 256; ++s) {
        window_sum += hist[s + ZS_WINDOW - 1] - hist[s - 1];
        if (window_sum > best_sum) { // strict: the smallest start wins a tie
            best_sum = window_sum;
            win_lo = s;
        }
    }
    const int base_exp = win_lo - 1;

    // ---- pass 2: in-window count of every BlockTile -> segment offsets
    std::vector<uint32_t> n_high_bt(n_bt);
    for_each_strip(n_strips, threads, [&](int64_t strip, int) {
        for (int64_t kb = 0; kb < bts_per_strip; ++kb) {
            uint32_t c = 0;
            for (int r = 0; r < ZS_BT_DIM; ++r) {
                const uint16_t *row = W + (strip * ZS_BT_DIM + r) * ldw + kb * ZS_BT_DIM;
                for (int k = 0; k < ZS_BT_DIM; ++k) c += in_window(row[k], (unsigned)win_lo);
            }
            n_high_bt[(size_t)(strip * bts_per_strip + kb)] = c;
        }
    });

    Sections sec;
    sec.off_bitmaps = 0;
    sec.off_offsets = align_up(n_bt * ZS_BT_BITMAP_BYTES, ZS_SECTION_ALIGN);
    sec.off_H = align_up(sec.off_offsets + (n_bt + 1) * 8, ZS_SECTION_ALIGN);
    uint8_t *base = static_cast<uint8_t *>(blob);
    uint32_t *offsets = reinterpret_cast<uint32_t *>(base + sec.off_offsets);
    uint64_t h_units = 0, l_units = 0, n_high = 0;
    uint32_t max_h = 0, max_l = 0;
    for (uint64_t bt = 0; bt < n_bt; ++bt) {
        offsets[2 * bt + 0] = (uint32_t)h_units;
        offsets[2 * bt + 1] = (uint32_t)l_units;
        uint32_t nh = n_high_bt[bt], nl = ZS_BT_ELEMS - nh;
        uint32_t hu = (nh + 15) / 16, lu = (2 * nl + 15) / 16;
        max_h = std::max(max_h, hu);
        max_l = std::max(max_l, lu);
        h_units += hu;
        l_units += lu;
        n_high += nh;
    }
    offsets[2 * n_bt + 0] = (uint32_t)h_units;
    offsets[2 * n_bt + 1] = (uint32_t)l_units;
    {
        // zero the tail of the offsets section up to the next section
        uint64_t end = sec.off_offsets + (n_bt + 1) * 8;
        std::memset(base + end, 0, (size_t)(sec.off_H - end));
        uint64_t bend = n_bt * ZS_BT_BITMAP_BYTES;
        std::memset(base + bend, 0, (size_t)(sec.off_offsets - bend));
    }
    sec.off_L = align_up(sec.off_H + h_units * 16, ZS_SECTION_ALIGN);
    const uint64_t total = align_up(sec.off_L + l_units * 16, ZS_SECTION_ALIGN);
    if (total > blob_cap) return ZS_ERR_SIZE;
    std::memset(base + sec.off_H + h_units * 16, 0, (size_t)(sec.off_L - (sec.off_H + h_units * 16)));
    std::memset(base + sec.off_L + l_units * 16, 0, (size_t)(total - (sec.off_L + l_units * 16)));

    // ---- pass 3: tile encoding (Algorithm 1, phase II)
    for_each_strip(n_strips, threads, [&](int64_t strip, int) {
        for (int64_t kb = 0; kb < bts_per_strip; ++kb) {
            const uint64_t bt = (uint64_t)(strip * bts_per_strip + kb);
            uint64_t *planes = reinterpret_cast<uint64_t *>(base + sec.off_bitmaps + bt * ZS_BT_BITMAP_BYTES);
            uint8_t *h = base + sec.off_H + (uint64_t)offsets[2 * bt] * 16;
            uint16_t *l = reinterpret_cast<uint16_t *>(base + sec.off_L + (uint64_t)offsets[2 * bt + 1] * 16);
            uint8_t *h_end = base + sec.off_H + (uint64_t)offsets[2 * bt + 2] * 16;
            uint16_t *l_end = reinterpret_cast<uint16_t *>(base + sec.off_L + (uint64_t)offsets[2 * bt + 3] * 16);
            const uint16_t *tile = W + strip * ZS_BT_DIM * ldw + kb * ZS_BT_DIM;
            for (int tt = 0; tt < ZS_TT_PER_BT; ++tt)
                for (int ft = 0; ft < ZS_FT_PER_TT; ++ft) {
                    int row0, col0;
                    fragtile_origin(tt, ft, row0, col0);
                    uint64_t plane[3] = {0, 0, 0};
                    for (int r = 0; r < 8; ++r) {
                        const uint16_t *src = tile + (row0 + r) * ldw + col0;
                        for (int c = 0; c < 8; ++c) {
                            const uint16_t w = src[c];
                            const unsigned d = ((w >> 7) & 0xFFu) - (unsigned)win_lo;
                            if (d < 7u) {
                                const uint64_t code = d + 1; // exponent - base_exp, 1..7
                                const int p = 8 * r + c;
                                plane[0] |= (code & 1) << p;
                                plane[1] |= ((code >> 1) & 1) << p;
                                plane[2] |= ((code >> 2) & 1) << p;
                                *h++ = (uint8_t)(((w >> 8) & 0x80u) | (w & 0x7Fu));
                            } else {
                                *l++ = w;
                            }
                        }
                    }
                    uint64_t *dst = planes + 3 * (tt * ZS_FT_PER_TT + ft);
                    dst[0] = plane[0];
                    dst[1] = plane[1];
                    dst[2] = plane[2];
                }
            while (h < h_end) *h++ = 0;
            while (l < l_end) *l++ = 0;
        }
    });

    std::memset(out, 0, sizeof *out);
    out->magic = ZS_MAGIC;
    out->version = ZS_FORMAT_VERSION;
    out->N = N;
    out->K = K;
    out->base_exp = base_exp;
    out->tile_cfg = ZS_TILE_CFG_FT8_TT16x32_BT64;
    out->n_high = n_high;
    out->n_fallback = (uint64_t)N * (uint64_t)K - n_high;
    out->off_bitmaps = sec.off_bitmaps;
    out->off_offsets = sec.off_offsets;
    out->off_H = sec.off_H;
    out->off_L = sec.off_L;
    out->h_bytes = h_units * 16;
    out->l_bytes = l_units * 16;
    out->total_bytes = total;
    out->max_h_units = max_h;
    out->max_l_units = max_l;
    return ZS_OK;
}
