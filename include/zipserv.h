/*
 * zipserv.h -- C ABI of the MI355X-native ZipGEMM library (libzipserv_hip.so).
 *
 * The library implements the hot path of ZipServ (ASPLOS'26): BF16 weights stored in
 * the Tensor-Core-Aware Triple Bitmap Encoding (TCA-TBE, Section 4.2) are decoded on
 * the fly inside a GEMM kernel (ZipGEMM, Section 4.3) or by a standalone decompression
 * kernel (Section 4.4).  Built for gfx950 only.
 *
 * Conventions
 *   - C = A * decode(W)^T with A [M, K] (M = tokens), W [N, K] (N = output features),
 *     C [M, N].  The paper writes Y = W X with M = output features and N = tokens
 *     (Section 2.1); only the letters differ.
 *   - BF16 values travel as uint16_t bit patterns.
 *   - Every function returns ZS_OK (0) or a negative zs_status; nothing throws.
 *   - The library never allocates or frees device memory and never creates streams:
 *     the caller owns every buffer and the stream.  "host" / "device" below say where a
 *     pointer must live.  Device entry points are asynchronous on the given stream.
 *   - No global mutable state: calls are thread-safe as long as their output buffers
 *     (and scratch buffers, where one is passed) are distinct.
 *
 * Blob layout (position independent: offsets only, the same bytes are valid on host
 * and device; the base must be 256-byte aligned).  Geometry, Section 4.2:
 *   FragTile       8 x 8 elements, element p = 8 * row + col (row along N, col along K);
 *                  three uint64 bit-planes, bit p of plane j (j = 1..3) = bit j-1 of
 *                  the 3-bit codeword of element p (000 = fallback, c = exponent - base_exp).
 *   TensorCoreTile 16 (N) x 32 (K) = 2 x 4 FragTiles, N-fastest ("column-major"): one
 *                  A-operand of v_mfma_f32_16x16x32_bf16, lane l <-> FragTile l / 8, row l % 8.
 *   BlockTile      64 x 64 = 4 (N) x 2 (K) TensorCoreTiles, N-fastest; BlockTiles are
 *                  ordered K-fastest inside a 64-row strip, strips by ascending N.
 *   sections       bitmaps : 24 bytes per FragTile (plane1, plane2, plane3), storage order;
 *                  offsets : (n_bt + 1) pairs of uint32 {start of BlockTile's H segment,
 *                            start of its L segment}, both in 16-byte units; last pair = totals;
 *                  H       : one byte sign << 7 | mantissa per in-window element, storage
 *                            order, every BlockTile's segment zero-padded to 16 bytes;
 *                  L       : raw BF16 of every out-of-window element, same order and padding.
 */
#ifndef ZIPSERV_H
#define ZIPSERV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZS_OK = 0,
    ZS_ERR_ARG = -1,    /* null pointer, misaligned blob, negative size            */
    ZS_ERR_SHAPE = -2,  /* N or K not a positive multiple of 64, ld too small, M<1 */
    ZS_ERR_SIZE = -3,   /* output or workspace buffer too small                    */
    ZS_ERR_FORMAT = -4, /* descriptor does not describe a valid blob               */
    ZS_ERR_HIP = -5,    /* a HIP runtime call failed (launch error)                */
    ZS_ERR_CONFIG = -6  /* unknown kernel configuration id                         */
} zs_status;

#define ZS_MAGIC 0x45425A53u /* "SZBE" little endian */
#define ZS_FORMAT_VERSION 1u
#define ZS_TILE_CFG_FT8_TT16x32_BT64 1u

/* Host-resident description of one encoded matrix, filled by zs_encode. */
typedef struct {
    uint32_t magic, version;
    int64_t N, K;              /* W is [N, K]; both multiples of 64                        */
    int32_t base_exp;          /* in [-1, 248]; window = base_exp + 1 .. base_exp + 7       */
    uint32_t tile_cfg;         /* ZS_TILE_CFG_*                                             */
    uint64_t n_high;           /* elements in H                                            */
    uint64_t n_fallback;       /* elements in L  (n_high + n_fallback == N * K)            */
    uint64_t off_bitmaps;      /* byte offsets of the four sections inside the blob        */
    uint64_t off_offsets;
    uint64_t off_H;
    uint64_t off_L;
    uint64_t h_bytes, l_bytes; /* padded section sizes                                     */
    uint64_t total_bytes;      /* size of the blob                                         */
    uint32_t max_h_units;      /* largest per-BlockTile H / L segment, in 16-byte units    */
    uint32_t max_l_units;
} zs_desc;

/* Upper bound of zs_encode's output for an N x K matrix (all elements fallback, plus
 * padding).  Returns 0 for an invalid shape. */
size_t zs_encode_bound(int64_t N, int64_t K);

/* Offline compressor (Algorithm 1; layout of Section 4.2; 16-byte padding of Section
 * 4.3.1).  Host only, integer only, deterministic, multi-threaded over BlockTiles.
 *   W_host    [N, K] BF16 bit patterns, row stride ldw >= K elements          (host, in)
 *   blob_host at least zs_encode_bound(N, K) bytes or ZS_ERR_SIZE             (host, out)
 *   out       descriptor                                                      (host, out)
 *   threads   worker threads, <= 0 means "as many as the machine has"
 * Window = the 7 consecutive exponents of largest coverage, smallest start on ties;
 * zeros, subnormals, Inf and NaN are ordinary bit patterns. */
int zs_encode(const uint16_t *W_host, int64_t N, int64_t K, int64_t ldw,
              void *blob_host, size_t blob_cap, zs_desc *out, int threads);

/* GPU-side packer: Algorithm 1 and Section 4.2 as zs_encode, for a matrix that already lies in
 * device memory (weights loaded or produced on the GPU).  The blob is byte for byte the one
 * zs_encode writes for the same matrix.
 *   W_dev     [N, K] BF16 bit patterns, row stride ldw >= K, ldw % 8 == 0, 16-byte aligned (device, in)
 *   blob_dev  256-byte aligned, at least zs_encode_bound(N, K) bytes or ZS_ERR_SIZE  (device, out)
 *   out       descriptor                                                             (host, out)
 *   workspace_dev  ZS_ENCODE_WORKSPACE_BYTES of scratch, 16-byte aligned, any contents (device)
 * Runs five small kernels on hip_stream and waits for the stream twice (the exponent histogram
 * and the section sizes are read back by the host): not for use under graph capture.  Bytes of
 * blob_dev beyond out->total_bytes are left as they were. */
#define ZS_ENCODE_WORKSPACE_BYTES ((size_t)4096)
int zs_encode_device(const uint16_t *W_dev, int64_t N, int64_t K, int64_t ldw, void *blob_dev,
                     size_t blob_cap, zs_desc *out, void *workspace_dev, size_t workspace_bytes,
                     void *hip_stream);

/* Checks a descriptor against itself (magic, shape, section offsets and sizes). */
int zs_desc_validate(const zs_desc *d);

/* Standalone decompression kernel (Section 4.4; per-lane logic of Algorithm 2).
 *   blob_dev  the encoded blob, 256-byte aligned                              (device, in)
 *   W_out_dev [N, K] BF16 bit patterns, row stride ldw >= K, 16-byte aligned  (device, out)
 * Bit-exact inverse of zs_encode. */
int zs_decompress(const zs_desc *d, const void *blob_dev, uint16_t *W_out_dev, int64_t ldw,
                  void *hip_stream);

/* Scratch bytes zs_gemm can use for (d, M): strip counters plus two partial tiles per workgroup
 * (a few MB at most; 0 for the configurations that do not use any). */
size_t zs_gemm_workspace(const zs_desc *d, int64_t M);

/* Fused decompression-GEMM (ZipGEMM, Section 4.3): C = A * decode(W)^T, BF16 inputs,
 * FP32 accumulation on the matrix cores, FP32 output; C is overwritten (no alpha/beta).
 * The decoded weights exist only in registers / LDS, never in HBM.
 *   A_dev  [M, K] BF16 bit patterns, row stride lda >= K, 16-byte aligned rows (device, in)
 *   C_dev  [M, N] float, row stride ldc >= N, 16-byte aligned rows             (device, out)
 *   M      >= 1, any integer
 *   workspace_dev / workspace_bytes  optional scratch, 256-byte aligned, at least
 *          zs_gemm_workspace(d, M) bytes, ZERO-FILLED by the caller before its first use.  A
 *          call leaves every byte of it zero again, so one buffer can serve every later call,
 *          for any matrix, as long as calls that share it do not overlap (same stream, or
 *          otherwise ordered) and nothing else writes to it in between: a kernel that finds
 *          stale bytes there does not fault or hang, but the strips of C that were cut between
 *          workgroups come out wrong.                                          (device, scratch)
 * The tiling is chosen from (M, N, K) (Section 4.3.1 split-K; Section 4.4 stage awareness).
 * The work split can cut a 64-row strip of W between workgroups.  With scratch memory the
 * partial sums of such a strip are parked there and added up by the workgroup that arrives
 * last, in one kernel.  With workspace_dev NULL (or too small, or a configuration that uses
 * none) the matching columns of C are first cleared by a second small kernel on the same
 * stream and then summed with FP32 atomics.  Either way the order in which the waves of a
 * workgroup add their partial sums is not fixed: the last bits of C can differ from run to
 * run. */
int zs_gemm(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
            float *C_dev, int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes,
            void *hip_stream);

/* ZipGEMM (Section 4.3) with the result rounded to BF16, the activation type of the models the
 * paper serves (Section 6.1): C[M,N] = bf16(A * decode(W)^T), FP32 accumulation, one rounding
 * to nearest even at the end (NaN stays NaN).  Arguments as for zs_gemm except
 *   C_dev  [M, N] BF16 bit patterns, row stride ldc >= N elements, ldc % 4 == 0, 16-byte aligned
 *   workspace_dev / workspace_bytes  REQUIRED whenever zs_gemm_workspace(d, M < 64 ? M : 64) is
 *          not zero (partial sums of strips shared between workgroups cannot be added on a BF16
 *          C): same buffer, same zero-fill-once contract as zs_gemm; ZS_ERR_SIZE without it.
 * Runs the skinny-M kernels only: more than 64 tokens are processed as 64-token panels, each a
 * full pass over the blob (a decode-stage entry point; for prefill use zs_linear and convert). */
int zs_gemm_bf16(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
                 uint16_t *C_dev, int64_t ldc, int64_t M, void *workspace_dev,
                 size_t workspace_bytes, void *hip_stream);

/* As zs_gemm, with the tiling forced: the low 8 bits of config are a configuration id (0 picks
 * automatically; ids are listed by zs_gemm_config_name()), the bits above them the number of
 * workgroups (0 = one per compute unit).  Meant for benchmarks and tests. */
int zs_gemm_ex(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
               float *C_dev, int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes,
               void *hip_stream, int config);
size_t zs_gemm_workspace_ex(const zs_desc *d, int64_t M, int config);
/* Name of configuration id (1 .. zs_gemm_num_configs()), NULL when out of range. */
const char *zs_gemm_config_name(int config);
int zs_gemm_num_configs(void);
/* The configuration zs_gemm would pick for (d, M). */
int zs_gemm_pick_config(const zs_desc *d, int64_t M);

/* Dense BF16 GEMM on uncompressed weights through hipBLASLt (comparison baseline, and the second
 * half of the decoupled pipeline of Section 4.4): C[M,N] (FP32) = A[M,K] * W[N,K]^T, BF16 bit
 * patterns in, FP32 accumulation.  All pointers device, 16-byte aligned; lda, ldw >= K, ldc >= N.
 * workspace_dev / workspace_bytes: optional scratch for hipBLASLt (split-K kernels).
 * algo: index into the algorithms hipBLASLt's heuristic returns for this shape, in its order
 * (0 .. zs_dense_gemm_algos() - 1; 0 is the library's own first choice and what zs_linear runs);
 * ZS_ERR_CONFIG when out of range.  The first call on a device
 * creates a hipBLASLt handle, the first call for a shape queries the heuristic (both are kept). */
int zs_dense_gemm(const uint16_t *A_dev, int64_t lda, const uint16_t *W_dev, int64_t ldw,
                  float *C_dev, int64_t ldc, int64_t M, int64_t N, int64_t K,
                  void *workspace_dev, size_t workspace_bytes, void *hip_stream, int algo);
/* Number of algorithms the heuristic offers for the shape (at most 16), or a negative zs_status. */
int zs_dense_gemm_algos(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldw, int64_t ldc,
                        size_t workspace_bytes);

/* Stage-aware linear layer (Section 4.4): C = A * decode(W)^T like zs_gemm, by whichever path is
 * faster for M tokens.  Decode-sized batches run the fused ZipGEMM kernels (ZS_PATH_FUSED);
 * beyond a measured crossover (more than 256 tokens; from 128 tokens on small layers) the
 * decoupled pipeline runs (ZS_PATH_DECOUPLED): zs_decompress into the workspace, then
 * zs_dense_gemm on the decompressed weights, so that the decompression cost is paid once for
 * all tokens.  zs_linear_path() tells which; zs_linear_workspace() how much
 * workspace that path needs (the fused path's is optional as for zs_gemm and must be zero-filled
 * once, and again after a decoupled call has used the same buffer; the decoupled path's is required: 2 N K bytes for the weights, rounded up to 256, plus
 * ZS_DENSE_WORKSPACE_BYTES, and need not be initialised).  ZS_ERR_SIZE if the decoupled path
 * gets less. */
#define ZS_PATH_FUSED 0
#define ZS_PATH_DECOUPLED 1
#define ZS_DENSE_WORKSPACE_BYTES ((size_t)32 << 20)
int zs_linear_path(const zs_desc *d, int64_t M);
size_t zs_linear_workspace(const zs_desc *d, int64_t M);
int zs_linear(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
              float *C_dev, int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes,
              void *hip_stream);

/* zs_gemm for callers that cannot allocate device memory or hand over a scratch buffer: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, checks, tiling choice and result as zs_gemm; the scratch memory of the skinny-M
 * kernel (strip counters and two partial tiles per workgroup) is a device array of 8 MiB + 4 KiB
 * inside the library, one copy per GPU the library runs on, held until the process ends.  The
 * call allocates and frees nothing (its first call on a device looks the array's address up).
 *   - ZS_ERR_SIZE if the launch would need more scratch than the array holds (more than 256
 *     workgroups: a device with more than 256 compute units).
 *   - Every call on a GPU shares that GPU's array: calls that overlap on one GPU (different
 *     streams, not otherwise ordered) race.  The array keeps the last call's contents; the
 *     call clears the part it uses with a small kernel of its own before the GEMM kernel.
 *   - M > 64 runs the kernels that need no scratch memory, exactly as zs_gemm does. */
int zs_gemm_noalloc(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda,
                    float *C_dev, int64_t ldc, int64_t M, void *hip_stream);

/* ---- Format variants -------------------------------------------------------------------
 * Section 4.2 ("The Choice of Codeword Length") weighs 2-, 3- and 4-bit codewords by
 * AverageBits(n) = r_n (n + 8) + (1 - r_n)(n + 16) and keeps n = 3.  These entry points write
 * and read the same encoding at any of the three lengths, so that the comparison can be
 * measured on a given matrix: n bit-planes per FragTile, codeword c in 1 .. 2^n - 1 = exponent
 * base_exp + c, 0 = fallback, window = the 2^n - 1 consecutive exponents of largest coverage
 * (smallest start on ties).  Two further switches are extensions that the paper does not have:
 *   base_mode  ZS_BASE_MATRIX  one window per matrix (the paper's)
 *              ZS_BASE_TILE    one per 64 x 64 BlockTile
 *              ZS_BASE_ROW     one per BlockTile row (64 elements): for weights whose rows
 *                              differ in scale, which a matrix-wide window covers badly
 *   dense_h    nonzero: every element owns its sign+mantissa byte at a fixed place (64 per
 *              FragTile, p-th byte = element p, zero for a fallback); only fallbacks go to L.
 *              Costs 8 (1 - r) more bits per element; the decoder needs no prefix count for H.
 * Variant blobs are a format of their own (never read by zs_gemm / zs_decompress).  Sections,
 * each 256-byte aligned, element and tile order as in the main format:
 *   planes  : 8 n bytes per FragTile (plane 1 .. plane n)
 *   offsets : (n_bt + 1) pairs of uint32 {H segment start, L segment start} in 16-byte units
 *   bases   : first exponent of the window (base_exp + 1), one byte per BlockTile
 *             (ZS_BASE_MATRIX, ZS_BASE_TILE) or 64 per BlockTile, by row (ZS_BASE_ROW)
 *   H, L    : as in the main format; with dense_h every H segment is 4096 bytes
 * With (n_planes 3, ZS_BASE_MATRIX, dense_h 0) planes, offsets, H and L hold the same bytes as
 * the sections of zs_encode's blob. */
#define ZS_BASE_MATRIX 0
#define ZS_BASE_TILE 1
#define ZS_BASE_ROW 2
#define ZS_VARIANT_MAGIC 0x56425A53u /* "SZBV" little endian */
typedef struct {
    uint32_t magic, version;
    int32_t n_planes;           /* 2, 3 or 4                                                */
    int32_t base_mode;          /* ZS_BASE_*                                                */
    int32_t dense_h;            /* 0 or 1                                                   */
    int32_t reserved;
    int64_t N, K;               /* both multiples of 64                                     */
    uint64_t n_high, n_fallback;
    uint64_t off_planes, off_offsets, off_bases, off_H, off_L; /* byte offsets in the blob  */
    uint64_t h_bytes, l_bytes;  /* padded section sizes                                     */
    uint64_t total_bytes;       /* size of the blob                                         */
} zs_variant_desc;

/* Upper bound of zs_variant_encode's output; 0 for an invalid shape or variant. */
size_t zs_variant_bound(int64_t N, int64_t K, int n_planes, int base_mode, int dense_h);

/* Host packer for a variant (Algorithm 1 with 2^n - 1 in place of 7).  Arguments as zs_encode.
 * ZS_ERR_CONFIG for an unknown variant. */
int zs_variant_encode(const uint16_t *W_host, int64_t N, int64_t K, int64_t ldw, int n_planes,
                      int base_mode, int dense_h, void *blob_host, size_t blob_cap,
                      zs_variant_desc *out, int threads);

/* Checks a variant descriptor against itself. */
int zs_variant_validate(const zs_variant_desc *d);

/* Decompression kernel for variant blobs (Algorithm 2 with n planes), bit-exact inverse of
 * zs_variant_encode.  A plain kernel for the format comparison, not tuned like zs_decompress.
 *   blob_dev  256-byte aligned, d->total_bytes bytes, less than 4 GiB or ZS_ERR_SIZE (device, in)
 *   W_out_dev [N, K] BF16 bit patterns, row stride ldw >= K, ldw % 8 == 0, 16-byte aligned (device, out)
 * Every read of the blob goes through a bounds-checked buffer descriptor of d->total_bytes: a
 * corrupt blob yields wrong values, never an access outside it. */
int zs_variant_decompress(const zs_variant_desc *d, const void *blob_dev, uint16_t *W_out_dev,
                          int64_t ldw, void *hip_stream);

/* Compute units of the current device, which the tiling choices above scale with (256, those of
 * one MI355X, when no device can be asked: the sizing queries also run without a GPU). */
int zs_compute_units(void);

const char *zs_strerror(int status);
int zs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZIPSERV_H */
