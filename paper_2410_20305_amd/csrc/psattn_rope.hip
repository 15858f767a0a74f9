// Rotary position embedding inside the attention op (paper Section 3.1: position ids are set
// so that every response sits where it would sit in the normal paired format, i.e. the
// rejected response restarts right behind the prompt).
//
// Where the rotation happens:
//   Q   in the forward kernel's registers when the query row is loaded (each query row is
//       loaded exactly once); the rotated row is saved for the backward, whose k-major pass
//       streams Q tiles straight from global memory into LDS and cannot rotate them on the way.
//   K   once per layer by the small streaming kernel below: a K row is re-read by every q-tile
//       and q-head that sees it, so rotating it inside the attention kernels would repeat the
//       work dozens of times, and the K tiles travel global -> LDS without passing registers.
//       With grouped-query attention K is 1/G of Q, so this is the cheap half of a RoPE pass.
//   dQ, dK  turned back (gradient w.r.t. the unrotated tensors) in the registers of the dQ and
//       dK/dV kernels just before they are stored.
// No pass over a Q-sized tensor is added; position ids come from the per-token descriptors of
// the block mask, so no position array is stored either.
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <vector>

#include "psattn_mfma_common.h"

struct psattn_rope {
    int32_t head_dim = 0;
    int32_t max_positions = 0;
    float theta = 0.f;
    int device = -1;
    float* d_table = nullptr;  // [max_positions][128]: cos[64] | sin[64]
};

namespace psattn {
namespace {
using namespace mma;

// one thread per (token, kv-head, 8 dims below 64): rotates them and their partners above 64
__global__ __launch_bounds__(256) void psattn_rope_k_bf16(DeviceMeta meta, int Hkv, const float* table, const uint16_t* K,
                                                           uint16_t* Kr) {
    const size_t idx = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
    const size_t n = static_cast<size_t>(meta.T) * Hkv * 8;
    if (idx >= n) return;
    const int chunk = static_cast<int>(idx & 7);
    const size_t row = idx >> 3;               // token * Hkv + head
    const int t = static_cast<int>(row / Hkv);
    const float* trow = table + static_cast<size_t>(rope_position(meta.tok[t], t)) * 128;
    Frag8 lo, hi;
    lo.u = *reinterpret_cast<const uint4*>(K + row * 128 + 8 * chunk);
    hi.u = *reinterpret_cast<const uint4*>(K + row * 128 + 64 + 8 * chunk);
    rope_frag8(lo, hi, trow, 8 * chunk);
    *reinterpret_cast<uint4*>(Kr + row * 128 + 8 * chunk) = lo.u;
    *reinterpret_cast<uint4*>(Kr + row * 128 + 64 + 8 * chunk) = hi.u;
}

int check_rope(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t head_dim) {
    if (!meta || !rope) return PSATTN_EINVAL;
    if (dt != PSATTN_BF16 || head_dim != 128 || rope->head_dim != 128) return PSATTN_EUNSUPPORTED;
    if (!meta->on_device) return PSATTN_ENODEVICE;
    if (meta->n_positions > rope->max_positions) return PSATTN_ELIMIT;
    return PSATTN_OK;
}

}  // namespace
}  // namespace psattn

extern "C" {

int psattn_rope_create(int32_t head_dim, float theta, int32_t max_positions, void* hip_stream, psattn_rope** out) {
    if (!out) return PSATTN_EINVAL;
    *out = nullptr;
    if (max_positions <= 0 || !(theta > 0.f)) return PSATTN_EINVAL;
    if (head_dim != 128) return PSATTN_EUNSUPPORTED;
    psattn_rope* r = new (std::nothrow) psattn_rope();
    if (!r) return PSATTN_ENOMEM;
    r->head_dim = head_dim;
    r->max_positions = max_positions;
    r->theta = theta;
    const size_t n = static_cast<size_t>(max_positions) * 128;
    std::vector<float> host;
    try {
        host.resize(n);
    } catch (const std::bad_alloc&) {
        delete r;
        return PSATTN_ENOMEM;
    }
    // angles in double: a float product position * frequency would lose the low bits of long positions
    double inv_freq[64];
    for (int i = 0; i < 64; ++i) inv_freq[i] = std::pow(static_cast<double>(theta), -2.0 * i / head_dim);
    for (int32_t p = 0; p < max_positions; ++p)
        for (int i = 0; i < 64; ++i) {
            const double a = static_cast<double>(p) * inv_freq[i];
            host[static_cast<size_t>(p) * 128 + i] = static_cast<float>(std::cos(a));
            host[static_cast<size_t>(p) * 128 + 64 + i] = static_cast<float>(std::sin(a));
        }
    if (hipGetDevice(&r->device) != hipSuccess || hipMalloc(reinterpret_cast<void**>(&r->d_table), n * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        delete r;
        return PSATTN_ENOMEM;
    }
    // the host vector dies with this call, so the copy has to be complete on return
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(r->d_table, host.data(), n * sizeof(float), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(r->d_table);
        delete r;
        return PSATTN_EHIP;
    }
    *out = r;
    return PSATTN_OK;
}

int psattn_rope_free(psattn_rope* rope) {
    if (!rope) return PSATTN_OK;
    int rc = PSATTN_OK;
    if (rope->d_table && hipFree(rope->d_table) != hipSuccess) rc = PSATTN_EHIP;
    delete rope;
    return rc;
}

int psattn_rope_k(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_kv_heads, int32_t head_dim,
                  const void* K, void* Kr, void* hip_stream) {
    int rc = psattn::check_rope(meta, rope, dt, head_dim);
    if (rc != PSATTN_OK) return rc;
    if (n_kv_heads <= 0) return PSATTN_EINVAL;
    if (meta->T == 0) return PSATTN_OK;
    if (!K || !Kr) return PSATTN_EINVAL;
    const size_t n = static_cast<size_t>(meta->T) * n_kv_heads * 8;
    const size_t grid = (n + 255) / 256;
    if (grid > 0x7fffffffu) return PSATTN_EUNSUPPORTED;
    psattn::psattn_rope_k_bf16<<<static_cast<unsigned>(grid), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(
        meta->dev, n_kv_heads, rope->d_table, static_cast<const uint16_t*>(K), static_cast<uint16_t*>(Kr));
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}

int psattn_fwd_rope(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
                    int32_t head_dim, float scale, const void* Q, const void* K, const void* V, void* O, float* LSE,
                    void* Qr, void* Kr, void* hip_stream) {
    int rc = psattn::check_rope(meta, rope, dt, head_dim);
    if (rc != PSATTN_OK) return rc;
    if (!psattn_uses_mfma(meta, dt, head_dim, scale, 0)) return PSATTN_EUNSUPPORTED;
    if (meta->T > 0 && !Kr) return PSATTN_EINVAL;
    rc = psattn_rope_k(meta, rope, dt, n_kv_heads, head_dim, K, Kr, hip_stream);
    if (rc != PSATTN_OK) return rc;
    return psattn::fwd_checked(meta, dt, n_q_heads, n_kv_heads, head_dim, scale, Q, Kr, V, O, LSE, rope->d_table, Qr,
                               hip_stream);
}

int psattn_bwd_rope(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
                    int32_t head_dim, float scale, const void* Qr, const void* Kr, const void* V, const void* O,
                    const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    const int rc = psattn::check_rope(meta, rope, dt, head_dim);
    if (rc != PSATTN_OK) return rc;
    return psattn::bwd_checked(meta, dt, n_q_heads, n_kv_heads, head_dim, scale, Qr, Kr, V, O, dO, LSE, dQ, dK, dV,
                               workspace, workspace_bytes, hip_stream, rope->d_table);
}

}  // extern "C"
