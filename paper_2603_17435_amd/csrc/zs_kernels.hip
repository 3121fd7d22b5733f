// HIP kernels and device entry points of libzipserv_hip.so (gfx950 only).
//   zs_decompress : TCA-TBE blob -> row-major BF16 (standalone kernel, Section 4.4)
//   zs_gemm       : C = A * decode(W)^T, decode fused into the MFMA loop (ZipGEMM, Section 4.3)
#include <hip/hip_runtime.h>

#include "zipserv.h"
#include "zs_device.h"

using namespace zs;

namespace {

constexpr int kWavesPerWg = 4;
constexpr int kThreads = 64 * kWavesPerWg;
constexpr uint32_t kLdsBytes = kTableBytes + kWavesPerWg * kSlotBytes;

// --------------------------------------------------------------------------------------
// Standalone decompression.  One wave per BlockTile (grid-stride over BlockTiles): stage the
// tile in LDS, decode its eight TensorCoreTiles, store 16 bytes (8 weights) per lane.
// --------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void decompress_kernel(BlobView bv, uint16_t *out, int64_t ldw)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables<kNatural>(smem, bv.base_exp);
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t slot = kTableBytes + wave * kSlotBytes;
    const bool base_m1 = bv.base_exp < 0;
    const uint32_t n_bt = (uint32_t)bv.strips * (uint32_t)bv.k_blocks;
    const uint32_t row_in_tt = ((lane >> 3) & 1u) * 8u + (lane & 7u); // FragTiles run N-fastest
    const uint32_t col_in_tt = (lane >> 4) * 8u;

    for (uint32_t bt = blockIdx.x * kWavesPerWg + wave; bt < n_bt; bt += gridDim.x * kWavesPerWg) {
        Cursor cur = stage_block_tile(bv, bt, smem, slot, lane);
        __builtin_amdgcn_wave_barrier();
        const uint32_t strip = bt / (uint32_t)bv.k_blocks, kb = bt % (uint32_t)bv.k_blocks;
#pragma unroll 2
        for (int tt = 0; tt < ZS_TT_PER_BT; ++tt) {
            const u32x4 w = decode_tt<kNatural>(smem, 0, slot, tt, cur, lane, base_m1);
            const int64_t n = (int64_t)strip * 64 + (tt & 3) * 16 + row_in_tt;
            const int64_t k = (int64_t)kb * 64 + (tt >> 2) * 32 + col_in_tt;
            *reinterpret_cast<u32x4 *>(out + n * ldw + k) = w;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// --------------------------------------------------------------------------------------
// ZipGEMM, skinny-M regime.  W is the MFMA A operand (rows = output features), the
// activations are the B operand (columns = tokens, padded to MT * 16).  One wave owns a
// run of BlockTiles along K inside one 64-row strip: per BlockTile it stages the compressed
// bytes in LDS, decodes 8 TensorCoreTiles straight into operand registers and issues
// MT MFMAs per tile.  With split-K the partial sums are added to a zeroed C with FP32
// atomics, otherwise each wave stores its 64 x M block.
// --------------------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(kThreads) void gemm_skinny_kernel(BlobView bv, const uint16_t *A, int64_t lda,
                                                                float *C, int64_t ldc, int M, int k_splits)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    build_tables<kMfma>(smem, bv.base_exp);
    __syncthreads();

    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t slot = kTableBytes + wave * kSlotBytes;
    const bool base_m1 = bv.base_exp < 0;
    const uint32_t n_tasks = (uint32_t)bv.strips * (uint32_t)k_splits;
    const uint32_t m_lane = lane & 15u, kgrp = lane >> 4;

    for (uint32_t task = blockIdx.x * kWavesPerWg + wave; task < n_tasks; task += gridDim.x * kWavesPerWg) {
        const uint32_t strip = task / (uint32_t)k_splits, ks = task % (uint32_t)k_splits;
        const uint32_t kb0 = (uint32_t)(((uint64_t)bv.k_blocks * ks) / (uint32_t)k_splits);
        const uint32_t kb1 = (uint32_t)(((uint64_t)bv.k_blocks * (ks + 1)) / (uint32_t)k_splits);

        f32x4 acc[4][MT];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (uint32_t kb = kb0; kb < kb1; ++kb) {
            const uint32_t bt = strip * (uint32_t)bv.k_blocks + kb;
            Cursor cur = stage_block_tile(bv, bt, smem, slot, lane);

            // activations of this 64-wide K slab: lane (token m, k-group g) takes 8 consecutive k,
            // reordered to the (0,2)(1,3)(4,6)(5,7) element order of the decoded weights
            bf16x8 bop[2][MT];
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int j = 0; j < MT; ++j) {
                    const int m = j * 16 + (int)m_lane;
                    u32x4 a = u32x4{0u, 0u, 0u, 0u};
                    if (m < M)
                        a = *reinterpret_cast<const u32x4 *>(A + (int64_t)m * lda + (int64_t)kb * 64 + kh * 32 + kgrp * 8);
                    u32x4 p;
                    p.x = __builtin_amdgcn_perm(a.y, a.x, 0x05040100u);
                    p.y = __builtin_amdgcn_perm(a.y, a.x, 0x07060302u);
                    p.z = __builtin_amdgcn_perm(a.w, a.z, 0x05040100u);
                    p.w = __builtin_amdgcn_perm(a.w, a.z, 0x07060302u);
                    bop[kh][j] = __builtin_bit_cast(bf16x8, p);
                }
            __builtin_amdgcn_wave_barrier();

#pragma unroll
            for (int tt = 0; tt < ZS_TT_PER_BT; ++tt) {
                const u32x4 w = decode_tt<kMfma>(smem, 0, slot, tt, cur, lane, base_m1);
                const bf16x8 wop = __builtin_bit_cast(bf16x8, w);
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[tt & 3][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wop, bop[tt >> 2][j], acc[tt & 3][j], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
        }

        // D layout of the 16x16 MFMA: lane holds column (token) lane % 16, rows 4 * (lane / 16) + v
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const int m = j * 16 + (int)m_lane;
            if (m < M) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float *dst = C + (int64_t)m * ldc + (int64_t)strip * 64 + i * 16 + kgrp * 4;
                    if (k_splits == 1) {
                        *reinterpret_cast<f32x4 *>(dst) = acc[i][j];
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) unsafeAtomicAdd(dst + v, acc[i][j][v]);
                    }
                }
            }
        }
    }
}

__global__ void zero_rows_kernel(float *C, int64_t ldc, int M, int64_t N)
{
    const int64_t n4 = N / 4;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n4 * M; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = i / n4, c = i % n4;
        *reinterpret_cast<f32x4 *>(C + m * ldc + c * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// --------------------------------------------------------------------------------------
// Host side
// --------------------------------------------------------------------------------------
constexpr int kNumCus = 256;

int make_view(const zs_desc *d, const void *blob, BlobView *bv)
{
    if (!d || !blob) return ZS_ERR_ARG;
    int rc = zs_desc_validate(d);
    if (rc != ZS_OK) return rc;
    if (reinterpret_cast<uintptr_t>(blob) % ZS_SECTION_ALIGN) return ZS_ERR_ARG;
    if (d->K / 64 > INT32_MAX || d->N / 64 > INT32_MAX) return ZS_ERR_SHAPE;
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

struct GemmConfig {
    const char *name;
    int mt;       // tokens covered = 16 * mt
    int k_splits; // 0 = choose from the shape
};

// id 1..: fixed configurations for benchmarks; id 0 = automatic
const GemmConfig kConfigs[] = {
    {"skinny_m16_auto", 1, 0}, {"skinny_m32_auto", 2, 0}, {"skinny_m64_auto", 4, 0},
    {"skinny_m16_k1", 1, 1},   {"skinny_m16_k2", 1, 2},   {"skinny_m16_k4", 1, 4},
    {"skinny_m16_k8", 1, 8},   {"skinny_m16_k16", 1, 16}, {"skinny_m32_k1", 2, 1},
    {"skinny_m32_k4", 2, 4},   {"skinny_m32_k8", 2, 8},
};
constexpr int kNumConfigs = (int)(sizeof(kConfigs) / sizeof(kConfigs[0]));

int auto_k_splits(const zs_desc *d)
{
    // enough (strip, K-run) tasks to give every CU about 12 waves, but runs of >= 2 BlockTiles
    const int64_t strips = d->N / 64, kb = d->K / 64;
    int64_t want = (int64_t)kNumCus * 12;
    int64_t ks = (want + strips - 1) / strips;
    if (ks < 1) ks = 1;
    if (ks > kb / 2) ks = kb / 2 > 0 ? kb / 2 : 1;
    return (int)ks;
}

template <int MT>
int launch_skinny(const BlobView &bv, const uint16_t *A, int64_t lda, float *C, int64_t ldc, int M, int64_t N,
                  int k_splits, hipStream_t s)
{
    if (k_splits > 1) {
        const int64_t n = (int64_t)M * (N / 4);
        const int blocks = (int)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
        hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks), dim3(256), 0, s, C, ldc, M, N);
    }
    const int64_t tasks = (int64_t)bv.strips * k_splits;
    int64_t wgs = (tasks + kWavesPerWg - 1) / kWavesPerWg;
    const int64_t max_wgs = (int64_t)kNumCus * 3; // 3 workgroups of 53 KB LDS fit one CU
    if (wgs > max_wgs) wgs = max_wgs;
    hipLaunchKernelGGL(gemm_skinny_kernel<MT>, dim3((unsigned)wgs), dim3(kThreads), kLdsBytes, s, bv, A, lda, C,
                       ldc, M, k_splits);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
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
    int64_t wgs = (n_bt + kWavesPerWg - 1) / kWavesPerWg;
    const int64_t max_wgs = (int64_t)kNumCus * 3 * 4;
    if (wgs > max_wgs) wgs = max_wgs;
    hipLaunchKernelGGL(decompress_kernel, dim3((unsigned)wgs), dim3(kThreads), kLdsBytes,
                       static_cast<hipStream_t>(hip_stream), bv, W_out_dev, ldw);
    return hipGetLastError() == hipSuccess ? ZS_OK : ZS_ERR_HIP;
}

extern "C" int zs_gemm_num_configs(void) { return kNumConfigs; }

extern "C" const char *zs_gemm_config_name(int config)
{
    return (config >= 1 && config <= kNumConfigs) ? kConfigs[config - 1].name : nullptr;
}

extern "C" int zs_gemm_pick_config(const zs_desc *d, int64_t M)
{
    if (!d || M < 1) return 0;
    if (M <= 16) return 1;
    if (M <= 32) return 2;
    return 3;
}

extern "C" size_t zs_gemm_workspace_ex(const zs_desc *, int64_t, int) { return 0; }
extern "C" size_t zs_gemm_workspace(const zs_desc *d, int64_t M) { return zs_gemm_workspace_ex(d, M, 0); }

extern "C" int zs_gemm_ex(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                          int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream,
                          int config)
{
    (void)workspace_dev;
    (void)workspace_bytes;
    BlobView bv;
    int rc = make_view(d, blob_dev, &bv);
    if (rc != ZS_OK) return rc;
    if (!A_dev || !C_dev) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(A_dev) % 16 || reinterpret_cast<uintptr_t>(C_dev) % 16) return ZS_ERR_ARG;
    if (M < 1 || M > (1 << 20) || lda < d->K || lda % 8 || ldc < d->N || ldc % 4) return ZS_ERR_SHAPE;
    if (config == 0) config = zs_gemm_pick_config(d, M);
    if (config < 1 || config > kNumConfigs) return ZS_ERR_CONFIG;
    const GemmConfig &cfg = kConfigs[config - 1];
    const int k_splits = cfg.k_splits > 0 ? (cfg.k_splits <= d->K / 64 ? cfg.k_splits : (int)(d->K / 64))
                                          : auto_k_splits(d);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // tokens beyond the configuration's width are handled in successive column panels
    const int width = 16 * cfg.mt;
    for (int64_t m0 = 0; m0 < M; m0 += width) {
        const int m = (int)((M - m0) < width ? (M - m0) : width);
        const uint16_t *Ap = A_dev + m0 * lda;
        float *Cp = C_dev + m0 * ldc;
        switch (cfg.mt) {
        case 1: rc = launch_skinny<1>(bv, Ap, lda, Cp, ldc, m, d->N, k_splits, s); break;
        case 2: rc = launch_skinny<2>(bv, Ap, lda, Cp, ldc, m, d->N, k_splits, s); break;
        default: rc = launch_skinny<4>(bv, Ap, lda, Cp, ldc, m, d->N, k_splits, s); break;
        }
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
