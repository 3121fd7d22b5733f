/*
 * CPU oracle for the ZipServ hot path (TCA-TBE encode / decode, reference GEMM).
 *
 * THIS IS TEST INFRASTRUCTURE.  It defines what the HIP path must compute and is
 * called only from tests/, from __graft_entry__.smoke() and from the cpu_baseline
 * leg of bench.py.  It shares no code, header, table or constant with the HIP
 * library; the product never links, imports or calls it.
 *
 * Everything here is scalar, one element at a time, in the order the paper states
 * it.  Integer work is exact; the GEMM accumulates in double in ascending k.
 *
 * Paper passages followed (ZipServ, ASPLOS'26):
 *   - Algorithm 1 (offline compressor): histogram, window of 7 consecutive
 *     exponents, base_exp = min(window) - 1, per-tile bit-planes + H + L.
 *   - Section 4.2 (TCA-TBE): 3-bit codeword, three 64-bit bit-plane bitmaps per
 *     8x8 FragTile, PackedSignMantissa / FullValue buffers, Offset array,
 *     FragTile < TensorCoreTile < BlockTile nesting, FragTiles column-major in a
 *     TensorCoreTile; AverageBits(n) storage-cost formula.
 *   - Section 4.3.1: H and L segments padded to 128-bit alignment.
 *   - Algorithm 2 (thread-local decompression): spatial indicator, popcount
 *     addressing, implicit lookup e = base_exp + code.
 *   - Section 2.1: Y = W X (here C = A W^T with M = tokens, N = out features).
 *
 * Readings taken where the paper is silent (each is also listed in the design
 * document of this repository):
 *   - window = sliding 7-wide window of maximal coverage, ties -> smallest start;
 *     start may be 0, so base_exp is signed and lies in [-1, 248];
 *   - bit p of a bitmap (LSB = 0) <-> tile element p, p = 8*row + col, row along
 *     N (output features), col along K;
 *   - Pack(sign, mantissa) = sign << 7 | mantissa;
 *   - plane 1 holds code bit 0 (LSB), plane 3 holds code bit 2;
 *   - TensorCoreTile = 16 (N) x 32 (K) = 2 x 4 FragTiles, N-fastest
 *     ("column-major"); BlockTile = 64 x 64 = 4 (N) x 2 (K) TensorCoreTiles,
 *     N-fastest; BlockTiles K-fastest inside a 64-row strip, strips ascending;
 *   - "GroupTile" of the Offset array = BlockTile; offsets counted in 16-byte
 *     units; H and L of every BlockTile zero-padded to a multiple of 16 bytes;
 *   - no special-casing of zeros, subnormals, Inf or NaN.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ZSO_OK 0
#define ZSO_ERR_SHAPE (-1)
#define ZSO_ERR_CAP (-2)
#define ZSO_ERR_FORMAT (-3)

/* ---- BF16 field access (Section 2.2: 1 sign, 8 exponent, 7 mantissa bits) ---- */
static unsigned bf16_exponent(uint16_t w) { return (w >> 7) & 0xFFu; }
static unsigned bf16_sign(uint16_t w) { return (w >> 15) & 1u; }
static unsigned bf16_mantissa(uint16_t w) { return w & 0x7Fu; }

/* BF16 -> double, exact: BF16 is the upper half of an IEEE binary32. */
static double bf16_to_double(uint16_t w)
{
    uint32_t bits = ((uint32_t)w) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* ---- Algorithm 1, phase I ------------------------------------------------ */

/* 256-bin histogram of the exponent field over every element, no exclusions. */
void zso_exponent_histogram(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, uint64_t hist[256])
{
    for (int i = 0; i < 256; ++i) hist[i] = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            hist[bf16_exponent(W[n * ldw + k])] += 1;
}

/* Start s of the window {s, ..., s+6} of seven consecutive exponents with the
 * largest coverage; the first (smallest) such s wins a tie.  s ranges over
 * 0..249 so the window stays inside 0..255. */
int zso_select_window(const uint64_t hist[256], uint64_t *coverage_out)
{
    int best_s = 0;
    uint64_t best_cov = 0;
    for (int s = 0; s <= 249; ++s) {
        uint64_t cov = 0;
        for (int j = 0; j < 7; ++j) cov += hist[s + j];
        if (s == 0 || cov > best_cov) {
            best_cov = cov;
            best_s = s;
        }
    }
    if (coverage_out) *coverage_out = best_cov;
    return best_s;
}

/* Section 4.2 storage cost for codeword length 3:
 * AverageBits(3) = r*(3+8) + (1-r)*(3+16), r = covered fraction. */
double zso_average_bits3(const uint64_t hist[256], int window_start)
{
    uint64_t total = 0, cov = 0;
    for (int i = 0; i < 256; ++i) total += hist[i];
    for (int j = 0; j < 7; ++j) cov += hist[window_start + j];
    double r = (double)cov / (double)total;
    return r * 11.0 + (1.0 - r) * 19.0;
}

/* ---- Tile hierarchy (Section 4.2, "Hierarchical Tiling Design") ---------- */

/* Coordinates (n, k) of element p of FragTile ft of TensorCoreTile tt of
 * BlockTile bt, for a matrix with K columns. */
static void element_coords(int64_t K, int64_t bt, int tt, int ft, int p, int64_t *n, int64_t *k)
{
    int64_t bts_per_strip = K / 64;
    int64_t strip = bt / bts_per_strip; /* 64-row strip            */
    int64_t kb = bt % bts_per_strip;    /* BlockTile inside strip  */
    int tt_n = tt % 4;                  /* N-fastest: 4 along N    */
    int tt_k = tt / 4;                  /*            2 along K    */
    int ft_n = ft % 2;                  /* N-fastest: 2 along N    */
    int ft_k = ft / 2;                  /*            4 along K    */
    int row = p / 8;
    int col = p % 8;
    *n = 64 * strip + 16 * tt_n + 8 * ft_n + row;
    *k = 64 * kb + 32 * tt_k + 8 * ft_k + col;
}

static uint64_t round_up16(uint64_t x) { return (x + 15u) & ~(uint64_t)15u; }

typedef struct {
    int64_t N, K;
    int32_t window_start; /* s*                            */
    int32_t base_exp;     /* s* - 1, in [-1, 248]          */
    uint64_t n_bt;        /* number of BlockTiles          */
    uint64_t n_high;      /* elements stored in H          */
    uint64_t n_fallback;  /* elements stored in L          */
    uint64_t h_bytes;     /* padded size of the H array    */
    uint64_t l_bytes;     /* padded size of the L array    */
} zso_info;

/* Pass 1: statistics and array sizes, so the caller can allocate. */
int zso_encode_sizes(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, zso_info *info)
{
    if (N <= 0 || K <= 0 || N % 64 || K % 64 || ldw < K) return ZSO_ERR_SHAPE;
    uint64_t hist[256];
    zso_exponent_histogram(W, N, K, ldw, hist);
    int s = zso_select_window(hist, NULL);
    info->N = N;
    info->K = K;
    info->window_start = s;
    info->base_exp = s - 1;
    info->n_bt = (uint64_t)(N / 64) * (uint64_t)(K / 64);
    info->n_high = info->n_fallback = 0;
    info->h_bytes = info->l_bytes = 0;
    for (uint64_t bt = 0; bt < info->n_bt; ++bt) {
        uint64_t nh = 0, nl = 0;
        for (int tt = 0; tt < 8; ++tt)
            for (int ft = 0; ft < 8; ++ft)
                for (int p = 0; p < 64; ++p) {
                    int64_t n, k;
                    element_coords(K, (int64_t)bt, tt, ft, p, &n, &k);
                    int e = (int)bf16_exponent(W[n * ldw + k]);
                    if (e >= s && e <= s + 6) nh++; else nl++;
                }
        info->n_high += nh;
        info->n_fallback += nl;
        info->h_bytes += round_up16(nh);
        info->l_bytes += round_up16(2 * nl);
    }
    return ZSO_OK;
}

/* Pass 2 (Algorithm 1, phase II): fill
 *   planes : 3 * 64 * n_bt uint64  (plane1, plane2, plane3 of FragTile 0, then FragTile 1, ...)
 *   H      : info.h_bytes bytes
 *   L      : info.l_bytes / 2 uint16
 *   offH, offL : n_bt + 1 uint32, start of each BlockTile's segment in 16-byte units,
 *                last entry = total. */
int zso_encode(const uint16_t *W, int64_t N, int64_t K, int64_t ldw, const zso_info *info,
               uint64_t *planes, uint8_t *H, uint16_t *L, uint32_t *offH, uint32_t *offL)
{
    if (N != info->N || K != info->K) return ZSO_ERR_SHAPE;
    const int s = info->window_start;
    const int base = info->base_exp;
    uint64_t hpos = 0; /* byte index into H      */
    uint64_t lpos = 0; /* halfword index into L  */
    for (uint64_t bt = 0; bt < info->n_bt; ++bt) {
        offH[bt] = (uint32_t)(hpos / 16);
        offL[bt] = (uint32_t)(2 * lpos / 16);
        for (int tt = 0; tt < 8; ++tt)
            for (int ft = 0; ft < 8; ++ft) {
                uint64_t b1 = 0, b2 = 0, b3 = 0;
                for (int p = 0; p < 64; ++p) {
                    int64_t n, k;
                    element_coords(K, (int64_t)bt, tt, ft, p, &n, &k);
                    uint16_t w = W[n * ldw + k];
                    int e = (int)bf16_exponent(w);
                    if (e >= s && e <= s + 6) {
                        unsigned c = (unsigned)(e - base); /* 1..7 */
                        b1 |= (uint64_t)((c >> 0) & 1u) << p;
                        b2 |= (uint64_t)((c >> 1) & 1u) << p;
                        b3 |= (uint64_t)((c >> 2) & 1u) << p;
                        H[hpos++] = (uint8_t)((bf16_sign(w) << 7) | bf16_mantissa(w));
                    } else {
                        L[lpos++] = w;
                    }
                }
                uint64_t f = (bt * 8 + (uint64_t)tt) * 8 + (uint64_t)ft;
                planes[3 * f + 0] = b1;
                planes[3 * f + 1] = b2;
                planes[3 * f + 2] = b3;
            }
        while (hpos % 16) H[hpos++] = 0;
        while ((2 * lpos) % 16) L[lpos++] = 0;
    }
    offH[info->n_bt] = (uint32_t)(hpos / 16);
    offL[info->n_bt] = (uint32_t)(2 * lpos / 16);
    if (hpos != info->h_bytes || 2 * lpos != info->l_bytes) return ZSO_ERR_FORMAT;
    return ZSO_OK;
}

/* ---- Algorithm 2 --------------------------------------------------------- */

static int popcount64(uint64_t x)
{
    int c = 0;
    while (x) { c += (int)(x & 1u); x >>= 1; }
    return c;
}

/* Index arithmetic of Algorithm 2 for element p of a tile with indicator M:
 * returns 1 and the H index if bit p is set, else 0 and the L index. */
int zso_tile_index(uint64_t M, int p, int *idx)
{
    uint64_t mask = (p == 0) ? 0 : (((uint64_t)1 << p) - 1);
    int idx_h = popcount64(M & mask);
    if ((M >> p) & 1u) { *idx = idx_h; return 1; }
    *idx = p - idx_h;
    return 0;
}

/* Decoder following Algorithm 2: every element computes its own index with a
 * masked popcount, independently of every other element of the tile. */
int zso_decode_popc(const uint64_t *planes, const uint8_t *H, const uint16_t *L,
                    const uint32_t *offH, const uint32_t *offL, int32_t base_exp,
                    int64_t N, int64_t K, uint16_t *Wout, int64_t ldw)
{
    if (N <= 0 || K <= 0 || N % 64 || K % 64 || ldw < K) return ZSO_ERR_SHAPE;
    uint64_t n_bt = (uint64_t)(N / 64) * (uint64_t)(K / 64);
    for (uint64_t bt = 0; bt < n_bt; ++bt) {
        uint64_t start_h = (uint64_t)offH[bt] * 16;    /* bytes     */
        uint64_t start_l = (uint64_t)offL[bt] * 16 / 2; /* halfwords */
        for (int tt = 0; tt < 8; ++tt)
            for (int ft = 0; ft < 8; ++ft) {
                uint64_t f = (bt * 8 + (uint64_t)tt) * 8 + (uint64_t)ft;
                uint64_t b1 = planes[3 * f + 0], b2 = planes[3 * f + 1], b3 = planes[3 * f + 2];
                uint64_t M = b1 | b2 | b3; /* spatial indicator */
                for (int p = 0; p < 64; ++p) {
                    int64_t n, k;
                    element_coords(K, (int64_t)bt, tt, ft, p, &n, &k);
                    int idx;
                    uint16_t w;
                    if (zso_tile_index(M, p, &idx)) {
                        unsigned c = (unsigned)((((b3 >> p) & 1u) << 2) | (((b2 >> p) & 1u) << 1) | ((b1 >> p) & 1u));
                        unsigned e = (unsigned)(base_exp + (int)c); /* implicit lookup */
                        uint8_t sm = H[start_h + (uint64_t)idx];
                        w = (uint16_t)(((unsigned)(sm & 0x80u) << 8) | (e << 7) | (sm & 0x7Fu));
                    } else {
                        w = L[start_l + (uint64_t)idx];
                    }
                    Wout[n * ldw + k] = w;
                }
                int nh = popcount64(M);
                start_h += (uint64_t)nh;
                start_l += (uint64_t)(64 - nh);
            }
    }
    return ZSO_OK;
}

/* Second decoder, no popcount: walk the elements of a BlockTile in storage
 * order with two running cursors.  Brute-force cross-check of the one above. */
int zso_decode_walk(const uint64_t *planes, const uint8_t *H, const uint16_t *L,
                    const uint32_t *offH, const uint32_t *offL, int32_t base_exp,
                    int64_t N, int64_t K, uint16_t *Wout, int64_t ldw)
{
    if (N <= 0 || K <= 0 || N % 64 || K % 64 || ldw < K) return ZSO_ERR_SHAPE;
    uint64_t n_bt = (uint64_t)(N / 64) * (uint64_t)(K / 64);
    for (uint64_t bt = 0; bt < n_bt; ++bt) {
        const uint8_t *h = H + (uint64_t)offH[bt] * 16;
        const uint16_t *l = L + (uint64_t)offL[bt] * 8;
        for (int tt = 0; tt < 8; ++tt)
            for (int ft = 0; ft < 8; ++ft) {
                uint64_t f = (bt * 8 + (uint64_t)tt) * 8 + (uint64_t)ft;
                for (int p = 0; p < 64; ++p) {
                    int64_t n, k;
                    element_coords(K, (int64_t)bt, tt, ft, p, &n, &k);
                    unsigned c = 0;
                    for (int j = 0; j < 3; ++j) c |= (unsigned)((planes[3 * f + (uint64_t)j] >> p) & 1u) << j;
                    uint16_t w;
                    if (c != 0) {
                        uint8_t sm = *h++;
                        w = (uint16_t)(((unsigned)(sm >> 7) << 15) | ((unsigned)(base_exp + (int)c) << 7) | (sm & 0x7Fu));
                    } else {
                        w = *l++;
                    }
                    Wout[n * ldw + k] = w;
                }
            }
    }
    return ZSO_OK;
}

/* ---- Reference GEMM (Section 2.1), C = A * W^T ---------------------------- */

/* C[m, j] = sum_k A[m,k] * W[rows[j], k] in double, ascending k;
 * S[m, j] = sum_k |A[m,k] * W[rows[j], k]|  (the tolerance scale).
 * rows == NULL means rows[j] = j.  Row-parallel over j when threads > 1. */
void zso_gemm_rows(const uint16_t *A, int64_t lda, const uint16_t *W, int64_t ldw,
                   int64_t M, int64_t K, const int64_t *rows, int64_t n_rows,
                   double *C, double *S, int64_t ldc, int threads)
{
#ifdef _OPENMP
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
#endif
    for (int64_t j = 0; j < n_rows; ++j) {
        int64_t n = rows ? rows[j] : j;
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0, sabs = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double prod = bf16_to_double(A[m * lda + k]) * bf16_to_double(W[n * ldw + k]);
                acc += prod;
                sabs += fabs(prod);
            }
            C[m * ldc + j] = acc;
            S[m * ldc + j] = sabs;
        }
    }
}

int zso_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
