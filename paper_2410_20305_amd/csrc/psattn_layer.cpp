// A whole self-attention layer on prefix-shared sequences: Q/K/V projections, rotary
// embedding with paired-format position ids, prefix-shared attention, output projection,
// forward and backward.  This is the "attention layer" micro-benchmark of the paper's
// Section 4.2: the projections are linear in the number of tokens, so sharing the prompt
// saves them as well as the quadratic attention part.
//
// The four projections and their gradients are plain dense GEMMs and go to rocBLAS
// (bf16 in, fp32 accumulate); everything between them is libpsattn's own kernels, called
// through its C ABI.  Separate shared library: libpsattn.so itself stays free of the BLAS
// dependency.  Weights follow the [out_features, in_features] row-major convention,
// y = x W^T.
#include <hip/hip_runtime.h>
#include <rocblas/rocblas.h>

#include <cstdint>
#include <new>

#include "psattn.h"
#include "psattn_layer.h"

struct psattn_layer {
    int32_t hidden = 0, Hq = 0, Hkv = 0, d = 0;
    rocblas_handle blas = nullptr;
};

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// activations and gradients kept between forward and backward, carved out of the caller's workspace
struct Slots {
    char *Q, *K, *V, *Qr, *Kr, *O, *dO, *dQ, *dK, *dV, *attn_ws;
    float* LSE;
    size_t attn_ws_bytes, total;
};

Slots carve(const psattn_layer* L, const psattn_meta* meta, int32_t T, void* base) {
    Slots s{};
    const size_t q = static_cast<size_t>(T) * L->Hq * L->d * 2, k = static_cast<size_t>(T) * L->Hkv * L->d * 2;
    char* p = reinterpret_cast<char*>(align_up(reinterpret_cast<uintptr_t>(base), 256));
    char* p0 = p;
    auto take = [&](size_t n) { char* r = p; p += align_up(n, 256); return r; };
    s.Q = take(q); s.K = take(k); s.V = take(k); s.Qr = take(q); s.Kr = take(k); s.O = take(q);
    s.dO = take(q); s.dQ = take(q); s.dK = take(k); s.dV = take(k);
    s.LSE = reinterpret_cast<float*>(take(static_cast<size_t>(T) * L->Hq * 4));
    s.attn_ws_bytes = psattn_bwd_workspace_bytes(meta, L->Hq, L->Hkv, L->d);
    s.attn_ws = take(s.attn_ws_bytes);
    s.total = static_cast<size_t>(p - p0) + 256;
    return s;
}

// row-major C[M x N] = op(A) op(B) (+ C if accumulate); bf16 operands and result, fp32 accumulation.
// A row-major matrix read as column-major is its transpose, so C^T = op(B)^T op(A)^T is the same
// call with the operands swapped and each operation flag kept.
int gemm_rm(rocblas_handle h, bool ta, bool tb, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
            const void* B, int64_t ldb, void* C, int64_t ldc, bool accumulate) {
    if (M == 0 || N == 0) return PSATTN_OK;
    if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return PSATTN_EUNSUPPORTED;
    const float alpha = 1.f, beta = accumulate ? 1.f : 0.f;
    const rocblas_status st = rocblas_gemm_ex(
        h, tb ? rocblas_operation_transpose : rocblas_operation_none, ta ? rocblas_operation_transpose : rocblas_operation_none,
        static_cast<rocblas_int>(N), static_cast<rocblas_int>(M), static_cast<rocblas_int>(K), &alpha, B,
        rocblas_datatype_bf16_r, static_cast<rocblas_int>(ldb), A, rocblas_datatype_bf16_r, static_cast<rocblas_int>(lda), &beta, C,
        rocblas_datatype_bf16_r, static_cast<rocblas_int>(ldc), C, rocblas_datatype_bf16_r, static_cast<rocblas_int>(ldc),
        rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    return st == rocblas_status_success ? PSATTN_OK : PSATTN_EHIP;
}

}  // namespace

extern "C" {

int psattn_layer_create(int32_t hidden, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, psattn_layer** out) {
    if (!out) return PSATTN_EINVAL;
    *out = nullptr;
    if (hidden <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0) return PSATTN_EINVAL;
    if (head_dim != 128) return PSATTN_EUNSUPPORTED;  // the rotary-embedding kernels
    psattn_layer* L = new (std::nothrow) psattn_layer();
    if (!L) return PSATTN_ENOMEM;
    L->hidden = hidden; L->Hq = n_q_heads; L->Hkv = n_kv_heads; L->d = head_dim;
    if (rocblas_create_handle(&L->blas) != rocblas_status_success) {
        delete L;
        return PSATTN_EHIP;
    }
    rocblas_set_pointer_mode(L->blas, rocblas_pointer_mode_host);
    *out = L;
    return PSATTN_OK;
}

int psattn_layer_free(psattn_layer* layer) {
    if (!layer) return PSATTN_OK;
    const bool ok = !layer->blas || rocblas_destroy_handle(layer->blas) == rocblas_status_success;
    delete layer;
    return ok ? PSATTN_OK : PSATTN_EHIP;
}

size_t psattn_layer_workspace_bytes(const psattn_layer* layer, const psattn_meta* meta, int32_t total_tokens) {
    if (!layer || !meta || total_tokens < 0) return 0;
    return carve(layer, meta, total_tokens, nullptr).total;
}

int psattn_layer_fwd(psattn_layer* L, const psattn_meta* meta, const psattn_rope* rope, int32_t total_tokens, float scale,
                     const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo, void* Y,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!L || !meta || !rope) return PSATTN_EINVAL;
    const int32_t T = total_tokens;
    if (T < 0) return PSATTN_EINVAL;
    if (T == 0) return PSATTN_OK;
    if (!X || !Wq || !Wk || !Wv || !Wo || !Y || !workspace) return PSATTN_EINVAL;
    if (workspace_bytes < psattn_layer_workspace_bytes(L, meta, T)) return PSATTN_EINVAL;
    if (rocblas_set_stream(L->blas, static_cast<hipStream_t>(hip_stream)) != rocblas_status_success) return PSATTN_EHIP;
    const Slots s = carve(L, meta, T, workspace);
    const int64_t h = L->hidden, nq = static_cast<int64_t>(L->Hq) * L->d, nk = static_cast<int64_t>(L->Hkv) * L->d;
    int rc;
    if ((rc = gemm_rm(L->blas, false, true, T, nq, h, X, h, Wq, h, s.Q, nq, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, false, true, T, nk, h, X, h, Wk, h, s.K, nk, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, false, true, T, nk, h, X, h, Wv, h, s.V, nk, false)) != PSATTN_OK) return rc;
    rc = psattn_fwd_rope(meta, rope, PSATTN_BF16, L->Hq, L->Hkv, L->d, scale, s.Q, s.K, s.V, s.O, s.LSE, s.Qr, s.Kr, hip_stream);
    if (rc != PSATTN_OK) return rc;
    return gemm_rm(L->blas, false, true, T, h, nq, s.O, nq, Wo, nq, Y, h, false);
}

int psattn_layer_bwd(psattn_layer* L, const psattn_meta* meta, const psattn_rope* rope, int32_t total_tokens, float scale,
                     const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo, const void* dY,
                     void* dX, void* dWq, void* dWk, void* dWv, void* dWo, void* workspace, size_t workspace_bytes,
                     void* hip_stream) {
    if (!L || !meta || !rope) return PSATTN_EINVAL;
    const int32_t T = total_tokens;
    if (T < 0) return PSATTN_EINVAL;
    if (!X || !Wq || !Wk || !Wv || !Wo || !dY || !dX || !dWq || !dWk || !dWv || !dWo || !workspace) return PSATTN_EINVAL;
    if (workspace_bytes < psattn_layer_workspace_bytes(L, meta, T)) return PSATTN_EINVAL;
    if (rocblas_set_stream(L->blas, static_cast<hipStream_t>(hip_stream)) != rocblas_status_success) return PSATTN_EHIP;
    const Slots s = carve(L, meta, T, workspace);
    const int64_t h = L->hidden, nq = static_cast<int64_t>(L->Hq) * L->d, nk = static_cast<int64_t>(L->Hkv) * L->d;
    int rc;
    // output projection: dO = dY Wo, dWo = dY^T O
    if ((rc = gemm_rm(L->blas, false, false, T, nq, h, dY, h, Wo, nq, s.dO, nq, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, true, false, h, nq, T, dY, h, s.O, nq, dWo, nq, false)) != PSATTN_OK) return rc;
    // attention: gradients w.r.t. the unrotated Q, K
    rc = psattn_bwd_rope(meta, rope, PSATTN_BF16, L->Hq, L->Hkv, L->d, scale, s.Qr, s.Kr, s.V, s.O, s.dO, s.LSE, s.dQ, s.dK,
                         s.dV, s.attn_ws, s.attn_ws_bytes, hip_stream);
    if (rc != PSATTN_OK) return rc;
    // projections: dW = dP^T X, dX = dQ Wq + dK Wk + dV Wv
    if ((rc = gemm_rm(L->blas, true, false, nq, h, T, s.dQ, nq, X, h, dWq, h, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, true, false, nk, h, T, s.dK, nk, X, h, dWk, h, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, true, false, nk, h, T, s.dV, nk, X, h, dWv, h, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, false, false, T, h, nq, s.dQ, nq, Wq, h, dX, h, false)) != PSATTN_OK) return rc;
    if ((rc = gemm_rm(L->blas, false, false, T, h, nk, s.dK, nk, Wk, h, dX, h, true)) != PSATTN_OK) return rc;
    return gemm_rm(L->blas, false, false, T, h, nk, s.dV, nk, Wv, h, dX, h, true);
}

}  // extern "C"
