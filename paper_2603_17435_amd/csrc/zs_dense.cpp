// Dense BF16 GEMM on uncompressed weights through the hipBLASLt C API, and the stage-aware
// entry point of Section 4.4 of the ZipServ paper: few tokens run the fused ZipGEMM kernel, many
// tokens run the decoupled pipeline (standalone decompression into caller-provided memory,
// then the vendor's dense GEMM), whose decompression cost is amortised over the tokens.
//
// hipBLASLt is the only thing here that keeps state: one handle per device and a small cache of
// the heuristic's algorithms per problem shape, both created on first use.
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>

#include <map>
#include <mutex>
#include <tuple>
#include <vector>

#include "zipserv.h"

namespace {

constexpr int kMaxDevices = 64;
constexpr int kMaxAlgos = 16;

struct Problem {
    int device;
    int64_t M, N, K, lda, ldw, ldc;
    size_t ws;
    bool operator<(const Problem &o) const
    {
        return std::tie(device, M, N, K, lda, ldw, ldc, ws) < std::tie(o.device, o.M, o.N, o.K, o.lda, o.ldw, o.ldc, o.ws);
    }
};

// Everything hipblasLtMatmul needs for one problem shape.
struct Plan {
    hipblasLtMatmulDesc_t op = nullptr;
    hipblasLtMatrixLayout_t w = nullptr, a = nullptr, c = nullptr;
    std::vector<hipblasLtMatmulHeuristicResult_t> algos;
};

std::mutex g_mutex;
hipblasLtHandle_t g_handle[kMaxDevices];
std::map<Problem, Plan> g_plans;

// Row-major C[M,N] = A[M,K] W[N,K]^T is, in hipBLASLt's column-major terms,
// C^T (N x M, ld ldc) = op_T(W as K x N, ld ldw) * (A as K x M, ld lda).
int plan_for(const Problem &p, Plan **out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    if (p.device < 0 || p.device >= kMaxDevices) return ZS_ERR_HIP;
    if (!g_handle[p.device] && hipblasLtCreate(&g_handle[p.device]) != HIPBLAS_STATUS_SUCCESS) return ZS_ERR_HIP;
    auto it = g_plans.find(p);
    if (it == g_plans.end()) {
        Plan pl;
        const hipblasOperation_t t = HIPBLAS_OP_T, n = HIPBLAS_OP_N;
        bool ok = hipblasLtMatmulDescCreate(&pl.op, HIPBLAS_COMPUTE_32F, HIP_R_32F) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatmulDescSetAttribute(pl.op, HIPBLASLT_MATMUL_DESC_TRANSA, &t, sizeof(t)) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatmulDescSetAttribute(pl.op, HIPBLASLT_MATMUL_DESC_TRANSB, &n, sizeof(n)) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&pl.w, HIP_R_16BF, (uint64_t)p.K, (uint64_t)p.N, p.ldw) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&pl.a, HIP_R_16BF, (uint64_t)p.K, (uint64_t)p.M, p.lda) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&pl.c, HIP_R_32F, (uint64_t)p.N, (uint64_t)p.M, p.ldc) == HIPBLAS_STATUS_SUCCESS;
        hipblasLtMatmulPreference_t pref = nullptr;
        ok = ok && hipblasLtMatmulPreferenceCreate(&pref) == HIPBLAS_STATUS_SUCCESS;
        const uint64_t ws = p.ws;
        ok = ok && hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &ws, sizeof(ws)) ==
                       HIPBLAS_STATUS_SUCCESS;
        if (ok) {
            pl.algos.resize(kMaxAlgos);
            int found = 0;
            if (hipblasLtMatmulAlgoGetHeuristic(g_handle[p.device], pl.op, pl.w, pl.a, pl.c, pl.c, pref, kMaxAlgos,
                                                pl.algos.data(), &found) != HIPBLAS_STATUS_SUCCESS)
                found = 0;
            pl.algos.resize(found > 0 ? found : 0);
            // keep only entries the heuristic marks valid and whose workspace fits what the caller has
            size_t kept = 0;
            for (const auto &r : pl.algos)
                if (r.state == HIPBLAS_STATUS_SUCCESS && r.workspaceSize <= p.ws) pl.algos[kept++] = r;
            pl.algos.resize(kept);
        }
        if (pref) hipblasLtMatmulPreferenceDestroy(pref);
        if (!ok || pl.algos.empty()) {
            if (pl.c) hipblasLtMatrixLayoutDestroy(pl.c);
            if (pl.a) hipblasLtMatrixLayoutDestroy(pl.a);
            if (pl.w) hipblasLtMatrixLayoutDestroy(pl.w);
            if (pl.op) hipblasLtMatmulDescDestroy(pl.op);
            return ZS_ERR_HIP;
        }
        it = g_plans.emplace(p, std::move(pl)).first;
    }
    *out = &it->second;
    return ZS_OK;
}

int check_dense_args(const uint16_t *A, int64_t lda, const uint16_t *W, int64_t ldw, float *C, int64_t ldc, int64_t M,
                     int64_t N, int64_t K)
{
    if (!A || !W || !C) return ZS_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(A) % 16 || reinterpret_cast<uintptr_t>(W) % 16 || reinterpret_cast<uintptr_t>(C) % 16)
        return ZS_ERR_ARG;
    if (M < 1 || N < 1 || K < 1 || lda < K || ldw < K || ldc < N) return ZS_ERR_SHAPE;
    return ZS_OK;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Tokens from which the decoupled pipeline is used.  Its cost is one decompression (the blob
// read and the BF16 matrix written, whatever M) plus the dense GEMM; the fused kernels pay their
// decode once per 256 tokens.  Measured on MI355X on the LLaMA-3 8B layer shapes: on the large
// layers (GateUp, Down) the fused kernels win up to 256 tokens and lose from 512 on; on the
// small ones (QKV, O: under 40 BlockTiles per compute unit), where the fused kernels are
// dominated by fixed costs, the switch pays from 128 tokens.
int64_t decoupled_from(const zs_desc *d)
{
    const int64_t tiles_per_cu = (d->N / 64) * (d->K / 64) / zs_compute_units();
    return tiles_per_cu < 40 ? 128 : 257;
}

} // namespace

extern "C" int zs_dense_gemm_algos(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldw, int64_t ldc,
                                   size_t workspace_bytes)
{
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return ZS_ERR_HIP;
    if (M < 1 || N < 1 || K < 1 || lda < K || ldw < K || ldc < N) return ZS_ERR_SHAPE;
    Plan *pl = nullptr;
    const int rc = plan_for(Problem{device, M, N, K, lda, ldw, ldc, workspace_bytes}, &pl);
    return rc == ZS_OK ? (int)pl->algos.size() : rc;
}

extern "C" int zs_dense_gemm(const uint16_t *A_dev, int64_t lda, const uint16_t *W_dev, int64_t ldw, float *C_dev,
                             int64_t ldc, int64_t M, int64_t N, int64_t K, void *workspace_dev, size_t workspace_bytes,
                             void *hip_stream, int algo)
{
    int rc = check_dense_args(A_dev, lda, W_dev, ldw, C_dev, ldc, M, N, K);
    if (rc != ZS_OK) return rc;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return ZS_ERR_HIP;
    if (!workspace_dev) workspace_bytes = 0;
    Plan *pl = nullptr;
    if ((rc = plan_for(Problem{device, M, N, K, lda, ldw, ldc, workspace_bytes}, &pl)) != ZS_OK) return rc;
    if (algo < 0 || algo >= (int)pl->algos.size()) return ZS_ERR_CONFIG;
    const float one = 1.f, zero = 0.f;
    const hipblasStatus_t st =
        hipblasLtMatmul(g_handle[device], pl->op, &one, W_dev, pl->w, A_dev, pl->a, &zero, C_dev, pl->c, C_dev, pl->c,
                        &pl->algos[algo].algo, workspace_dev, workspace_bytes, static_cast<hipStream_t>(hip_stream));
    return st == HIPBLAS_STATUS_SUCCESS ? ZS_OK : ZS_ERR_HIP;
}

extern "C" int zs_linear_path(const zs_desc *d, int64_t M)
{
    if (!d || M < 1 || zs_desc_validate(d) != ZS_OK) return -1;
    return M >= decoupled_from(d) ? ZS_PATH_DECOUPLED : ZS_PATH_FUSED;
}

extern "C" size_t zs_linear_workspace(const zs_desc *d, int64_t M)
{
    const int path = zs_linear_path(d, M);
    if (path < 0) return 0;
    if (path == ZS_PATH_FUSED) return zs_gemm_workspace(d, M);
    return align_up((size_t)d->N * (size_t)d->K * 2) + ZS_DENSE_WORKSPACE_BYTES;
}

extern "C" int zs_linear(const zs_desc *d, const void *blob_dev, const uint16_t *A_dev, int64_t lda, float *C_dev,
                         int64_t ldc, int64_t M, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    const int path = zs_linear_path(d, M);
    if (path < 0) return d ? (M < 1 ? ZS_ERR_SHAPE : zs_desc_validate(d)) : ZS_ERR_ARG;
    if (path == ZS_PATH_FUSED)
        return zs_gemm(d, blob_dev, A_dev, lda, C_dev, ldc, M, workspace_dev, workspace_bytes, hip_stream);
    // decoupled: TCA-TBE -> BF16 in the workspace, then the dense GEMM on it
    if (!workspace_dev || reinterpret_cast<uintptr_t>(workspace_dev) % kAlign) return ZS_ERR_ARG;
    if (workspace_bytes < zs_linear_workspace(d, M)) return ZS_ERR_SIZE;
    uint16_t *W = static_cast<uint16_t *>(workspace_dev);
    void *lt_ws = static_cast<uint8_t *>(workspace_dev) + align_up((size_t)d->N * (size_t)d->K * 2);
    int rc = zs_decompress(d, blob_dev, W, d->K, hip_stream);
    if (rc != ZS_OK) return rc;
    return zs_dense_gemm(A_dev, lda, W, d->K, C_dev, ldc, M, d->N, d->K, lt_ws, ZS_DENSE_WORKSPACE_BYTES, hip_stream, 0);
}
