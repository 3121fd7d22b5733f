// GPU-side TCA-TBE packer (Algorithm 1 and Section 4.2 of the ZipServ paper): the same blob,
// byte for byte, as the host packer zs_encode, from a matrix that already lies in device memory.
//
//   1. hist_kernel    exponent histogram                         -> host picks the window
//   2. count_kernel   in-window elements of every BlockTile      (parked in the offset section)
//   3. scan_kernel    segment offsets = prefix sums of the padded segment sizes, totals
//   4. pack_kernel    one wave per BlockTile: bit-planes, H bytes, L halfwords at their final
//                     place; fill_kernel zeroes the gaps between sections
// The host reads 2 KB after step 1 and 64 bytes after step 3 (two stream synchronisations): the
// window decides what is counted, the totals decide where the L section starts.
// Every store is checked against the caller's capacity, whatever the counts say.
#include <hip/hip_runtime.h>

#include <cstring>

#include "zipserv.h"
#include "zs_format.h"

namespace {

typedef uint32_t __attribute__((ext_vector_type(4))) u32x4;

constexpr int kHistWords = 256;                         // uint64 bins at the start of the workspace
constexpr size_t kTotalsAt = kHistWords * 8;            // then: struct Totals
struct Totals {
    uint64_t h_units, l_units, n_high;
    uint32_t max_h, max_l;
};
static_assert(kTotalsAt + sizeof(Totals) <= ZS_ENCODE_WORKSPACE_BYTES, "workspace layout");

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// The eight weights of FragTile row `lane` of TensorCoreTile tt of a BlockTile (the lane order of
// Section 4.2: lane l <-> FragTile l / 8, row l % 8), as 16 bytes.
__device__ __forceinline__ u32x4 load_row(const uint16_t *tile, int64_t ldw, int tt, uint32_t lane)
{
    const uint32_t ft = lane >> 3, r = lane & 7u;
    const uint32_t row = 16 * (tt & 3) + 8 * (ft & 1u) + r, col = 32 * (tt >> 2) + 8 * (ft >> 1);
    return *reinterpret_cast<const u32x4 *>(tile + (int64_t)row * ldw + col);
}
__device__ __forceinline__ uint32_t element(const u32x4 &v, int c)
{
    const uint32_t w = c < 2 ? v.x : c < 4 ? v.y : c < 6 ? v.z : v.w;
    return (c & 1) ? (w >> 16) : (w & 0xFFFFu);
}
__device__ __forceinline__ bool in_window(uint32_t w, uint32_t win_lo) { return ((w >> 7) & 0xFFu) - win_lo < 7u; }

// One workgroup of 256 threads per BlockTile; each thread sees 16 elements.
__global__ __launch_bounds__(256) void hist_kernel(const uint16_t *W, int64_t ldw, uint32_t k_blocks, unsigned long long *hist)
{
    __shared__ uint32_t bins[256];
    bins[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t bt = blockIdx.x, strip = bt / k_blocks, kb = bt % k_blocks;
    const uint16_t *tile = W + (int64_t)strip * 64 * ldw + (int64_t)kb * 64;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    for (int t = 0; t < 2; ++t) {
        const u32x4 v = load_row(tile, ldw, 2 * wave + t, lane);
#pragma unroll
        for (int c = 0; c < 8; ++c) atomicAdd(&bins[(element(v, c) >> 7) & 0xFFu], 1u);
    }
    __syncthreads();
    if (bins[threadIdx.x]) atomicAdd(&hist[threadIdx.x], (unsigned long long)bins[threadIdx.x]);
}

// In-window elements per BlockTile, written to the first word of the BlockTile's offset pair.
__global__ __launch_bounds__(256) void count_kernel(const uint16_t *W, int64_t ldw, uint32_t k_blocks, uint32_t win_lo,
                                                    uint32_t *offsets)
{
    __shared__ uint32_t total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    const uint32_t bt = blockIdx.x, strip = bt / k_blocks, kb = bt % k_blocks;
    const uint16_t *tile = W + (int64_t)strip * 64 * ldw + (int64_t)kb * 64;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t c_in = 0;
    for (int t = 0; t < 2; ++t) {
        const u32x4 v = load_row(tile, ldw, 2 * wave + t, lane);
#pragma unroll
        for (int c = 0; c < 8; ++c) c_in += in_window(element(v, c), win_lo) ? 1u : 0u;
    }
    atomicAdd(&total, c_in);
    __syncthreads();
    if (threadIdx.x == 0) offsets[2 * (size_t)bt] = total;
}

// One workgroup: offsets[bt] = {sum of H units before bt, sum of L units before bt}, in place over
// the counts left by count_kernel; offsets[n_bt] and the totals at the end.
__global__ __launch_bounds__(1024) void scan_kernel(uint32_t *offsets, uint32_t n_bt, Totals *totals)
{
    __shared__ uint32_t sh[1024], sl[1024];
    __shared__ uint64_t run_h, run_l, run_n;
    __shared__ uint32_t max_h, max_l;
    const uint32_t t = threadIdx.x;
    if (t == 0) run_h = 0, run_l = 0, run_n = 0, max_h = 0, max_l = 0;
    __syncthreads();
    for (uint32_t base = 0; base < n_bt; base += 1024) {
        const uint32_t bt = base + t;
        const bool live = bt < n_bt;
        const uint32_t nh = live ? offsets[2 * (size_t)bt] : 0u;
        const uint32_t hu = live ? (nh + 15u) / 16u : 0u, lu = live ? (2u * (ZS_BT_ELEMS - nh) + 15u) / 16u : 0u;
        sh[t] = hu, sl[t] = lu;
        __syncthreads();
        for (uint32_t d = 1; d < 1024; d <<= 1) { // inclusive scan of both arrays
            const uint32_t ah = t >= d ? sh[t - d] : 0u, al = t >= d ? sl[t - d] : 0u;
            __syncthreads();
            sh[t] += ah, sl[t] += al;
            __syncthreads();
        }
        if (live) {
            offsets[2 * (size_t)bt] = (uint32_t)(run_h + sh[t] - hu);
            offsets[2 * (size_t)bt + 1] = (uint32_t)(run_l + sl[t] - lu);
            atomicMax(&max_h, hu);
            atomicMax(&max_l, lu);
            atomicAdd((unsigned long long *)&run_n, (unsigned long long)nh);
        }
        __syncthreads();
        if (t == 0) run_h += sh[1023], run_l += sl[1023];
        __syncthreads();
    }
    if (t == 0) {
        offsets[2 * (size_t)n_bt] = (uint32_t)run_h;
        offsets[2 * (size_t)n_bt + 1] = (uint32_t)run_l;
        totals->h_units = run_h, totals->l_units = run_l, totals->n_high = run_n;
        totals->max_h = max_h, totals->max_l = max_l;
    }
}

__global__ void fill_kernel(uint8_t *p, uint64_t n)
{
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Exclusive prefix sum over the 64 lanes of a wave, and the wave total.
__device__ __forceinline__ uint32_t wave_exclusive(uint32_t x, uint32_t lane, uint32_t &total)
{
    uint32_t inc = x;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(inc, d, 64);
        if ((int)lane >= d) inc += up;
    }
    total = __shfl(inc, 63, 64);
    return inc - x;
}

// One wave per BlockTile.  A lane owns one FragTile row per TensorCoreTile: its byte of each
// bit-plane, its in-window bytes and its fallback halfwords, placed by prefix sums over the lanes.
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t *W, int64_t ldw, uint32_t k_blocks, uint32_t n_bt,
                                                   uint32_t win_lo, uint8_t *blob, uint64_t cap, uint64_t off_bitmaps,
                                                   const uint32_t *offsets, uint64_t off_H, uint64_t off_L)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t bt = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bt >= n_bt) return;
    const uint32_t strip = bt / k_blocks, kb = bt % k_blocks;
    const uint16_t *tile = W + (int64_t)strip * 64 * ldw + (int64_t)kb * 64;
    uint64_t h_at = off_H + (uint64_t)offsets[2 * (size_t)bt] * 16, l_at = off_L + (uint64_t)offsets[2 * (size_t)bt + 1] * 16;
    const uint64_t h_end = off_H + (uint64_t)offsets[2 * (size_t)bt + 2] * 16, l_end = off_L + (uint64_t)offsets[2 * (size_t)bt + 3] * 16;
    auto put8 = [&](uint64_t at, uint32_t v) {
        if (at < cap) blob[at] = (uint8_t)v;
    };
    auto put16 = [&](uint64_t at, uint32_t v) {
        if (at + 2 <= cap) *reinterpret_cast<uint16_t *>(blob + at) = (uint16_t)v;
    };
    for (int tt = 0; tt < ZS_TT_PER_BT; ++tt) {
        const u32x4 v = load_row(tile, ldw, tt, lane);
        uint32_t b1 = 0, b2 = 0, b3 = 0, n_in = 0;
        uint32_t hb[8], lw[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint32_t w = element(v, c), d = ((w >> 7) & 0xFFu) - win_lo;
            const bool in = d < 7u;
            const uint32_t code = in ? d + 1u : 0u; // exponent - base_exp, 1..7; 0 marks a fallback
            b1 |= (code & 1u) << c, b2 |= ((code >> 1) & 1u) << c, b3 |= ((code >> 2) & 1u) << c;
            hb[c] = ((w >> 8) & 0x80u) | (w & 0x7Fu);
            lw[c] = w;
            n_in += in ? 1u : 0u;
        }
        // byte r of a FragTile's 64-bit plane holds elements 8 r .. 8 r + 7: this lane's row
        const uint64_t planes = off_bitmaps + (uint64_t)bt * ZS_BT_BITMAP_BYTES + (uint64_t)(tt * ZS_FT_PER_TT + (lane >> 3)) * ZS_FT_BITMAP_BYTES + (lane & 7u);
        put8(planes, b1), put8(planes + 8, b2), put8(planes + 16, b3);
        uint32_t h_total, l_total;
        uint64_t h_pos = h_at + wave_exclusive(n_in, lane, h_total);
        uint64_t l_pos = l_at + 2ull * wave_exclusive(8u - n_in, lane, l_total);
        const uint32_t m = b1 | b2 | b3;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if ((m >> c) & 1u) put8(h_pos++, hb[c]);
            else put16(l_pos, lw[c]), l_pos += 2;
        }
        h_at += h_total, l_at += 2ull * l_total;
    }
    // padding up to the 16-byte boundary where the next BlockTile's segments start
    if (h_at + lane < h_end) put8(h_at + lane, 0);
    if (l_at + lane < l_end) put8(l_at + lane, 0);
}

} // namespace

extern "C" int zs_encode_device(const uint16_t *W_dev, int64_t N, int64_t K, int64_t ldw, void *blob_dev, size_t blob_cap,
                                zs_desc *out, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    if (!W_dev || !blob_dev || !out || !workspace_dev) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(W_dev) % 16 || reinterpret_cast<uintptr_t>(blob_dev) % ZS_SECTION_ALIGN ||
        reinterpret_cast<uintptr_t>(workspace_dev) % 16)
        return ZS_ERR_ARG;
    if (N <= 0 || K <= 0 || N % ZS_BT_DIM || K % ZS_BT_DIM || ldw < K || ldw % 8) return ZS_ERR_SHAPE;
    if (workspace_bytes < ZS_ENCODE_WORKSPACE_BYTES || blob_cap < zs_encode_bound(N, K)) return ZS_ERR_SIZE;
    const uint64_t n_bt64 = (uint64_t)(N / ZS_BT_DIM) * (uint64_t)(K / ZS_BT_DIM);
    if (n_bt64 >= (1ull << 31) || (uint64_t)N * (uint64_t)K / 8 >= (1ull << 32)) return ZS_ERR_SHAPE; // 32-bit unit offsets
    const uint32_t n_bt = (uint32_t)n_bt64, k_blocks = (uint32_t)(K / ZS_BT_DIM);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    uint8_t *blob = static_cast<uint8_t *>(blob_dev), *ws = static_cast<uint8_t *>(workspace_dev);
    unsigned long long *hist_dev = reinterpret_cast<unsigned long long *>(ws);
    Totals *totals_dev = reinterpret_cast<Totals *>(ws + kTotalsAt);
    auto ok = [](hipError_t e) { return e == hipSuccess; };

    // ---- window (Algorithm 1, phase I)
    hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(256), 0, s, ws, (uint64_t)ZS_ENCODE_WORKSPACE_BYTES);
    hipLaunchKernelGGL(hist_kernel, dim3(n_bt), dim3(256), 0, s, W_dev, ldw, k_blocks, hist_dev);
    uint64_t hist[kHistWords];
    if (!ok(hipGetLastError()) || !ok(hipMemcpyAsync(hist, hist_dev, sizeof hist, hipMemcpyDeviceToHost, s)) ||
        !ok(hipStreamSynchronize(s)))
        return ZS_ERR_HIP;
    uint64_t window_sum = 0;
    for (int j = 0; j < ZS_WINDOW; ++j) window_sum += hist[j];
    uint64_t best_sum = window_sum;
    int win_lo = 0;
    for (int st = 1; st + ZS_WINDOW <= 256; ++st) {
        window_sum += hist[st + ZS_WINDOW - 1] - hist[st - 1];
        if (window_sum > best_sum) best_sum = window_sum, win_lo = st; // strict: the smallest start wins a tie
    }

    // ---- segment offsets
    const uint64_t off_bitmaps = 0;
    const uint64_t off_offsets = align_up((uint64_t)n_bt * ZS_BT_BITMAP_BYTES, ZS_SECTION_ALIGN);
    const uint64_t off_H = align_up(off_offsets + ((uint64_t)n_bt + 1) * 8, ZS_SECTION_ALIGN);
    uint32_t *offsets_dev = reinterpret_cast<uint32_t *>(blob + off_offsets);
    hipLaunchKernelGGL(count_kernel, dim3(n_bt), dim3(256), 0, s, W_dev, ldw, k_blocks, (uint32_t)win_lo, offsets_dev);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, offsets_dev, n_bt, totals_dev);
    Totals tot;
    if (!ok(hipGetLastError()) || !ok(hipMemcpyAsync(&tot, totals_dev, sizeof tot, hipMemcpyDeviceToHost, s)) ||
        !ok(hipStreamSynchronize(s)))
        return ZS_ERR_HIP;
    const uint64_t off_L = align_up(off_H + tot.h_units * 16, ZS_SECTION_ALIGN);
    const uint64_t total = align_up(off_L + tot.l_units * 16, ZS_SECTION_ALIGN);
    if (total > blob_cap) return ZS_ERR_SIZE;

    // ---- gaps between the sections, then the tiles (Algorithm 1, phase II)
    auto zero = [&](uint64_t from, uint64_t to) {
        if (to > from) hipLaunchKernelGGL(fill_kernel, dim3(1), dim3(256), 0, s, blob + from, to - from);
    };
    zero((uint64_t)n_bt * ZS_BT_BITMAP_BYTES, off_offsets);
    zero(off_offsets + ((uint64_t)n_bt + 1) * 8, off_H);
    zero(off_H + tot.h_units * 16, off_L);
    zero(off_L + tot.l_units * 16, total);
    hipLaunchKernelGGL(pack_kernel, dim3((n_bt + 3) / 4), dim3(256), 0, s, W_dev, ldw, k_blocks, n_bt, (uint32_t)win_lo, blob,
                       (uint64_t)blob_cap, off_bitmaps, offsets_dev, off_H, off_L);
    if (!ok(hipGetLastError())) return ZS_ERR_HIP;

    std::memset(out, 0, sizeof *out);
    out->magic = ZS_MAGIC;
    out->version = ZS_FORMAT_VERSION;
    out->N = N;
    out->K = K;
    out->base_exp = win_lo - 1;
    out->tile_cfg = ZS_TILE_CFG_FT8_TT16x32_BT64;
    out->n_high = tot.n_high;
    out->n_fallback = (uint64_t)N * (uint64_t)K - tot.n_high;
    out->off_bitmaps = off_bitmaps;
    out->off_offsets = off_offsets;
    out->off_H = off_H;
    out->off_L = off_L;
    out->h_bytes = tot.h_units * 16;
    out->l_bytes = tot.l_units * 16;
    out->total_bytes = total;
    out->max_h_units = tot.max_h;
    out->max_l_units = tot.max_l;
    return ZS_OK;
}
