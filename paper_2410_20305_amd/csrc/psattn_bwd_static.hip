// psattn_bwd_static: psattn_bwd for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The backward
// scratch (delta and the rescaled LSE, two float arrays of n_q_heads * T entries) lives in
// a file-scope device array instead of a caller-provided workspace.
//
// Every device the library runs on holds its own copy of the array for the life of the
// process.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// address a kernel can use is looked up once per device (with that device current) and
// only that pointer is ever handed to kernels.
#include <hip/hip_runtime.h>

#include <mutex>

#include "psattn_internal.h"

namespace {

constexpr size_t kStaticRows = size_t{4} << 20;  // n_q_heads * T supported (config 5: 64 x 65 536)
constexpr size_t kStaticBytes = 2 * kStaticRows * sizeof(float) + 512;  // 32 MiB + alignment slack
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

std::mutex g_mu;
void* g_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device
int static_scratch(void** out) {
    *out = nullptr;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PSATTN_EHIP;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return PSATTN_EHIP;
        }
        g_ptr[dev] = p;
    }
    *out = g_ptr[dev];
    return PSATTN_OK;
}

}  // namespace

extern "C" {

size_t psattn_bwd_static_max_rows(void) { return kStaticRows; }

int psattn_bwd_static(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
                      int32_t head_dim, float scale, const void* Q, const void* K, const void* V,
                      const void* O, const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                      void* hip_stream) {
    if (!meta) return PSATTN_EINVAL;
    if (n_q_heads <= 0) return PSATTN_EINVAL;
    if (static_cast<size_t>(meta->T) * static_cast<size_t>(n_q_heads) > kStaticRows) return PSATTN_ELIMIT;
    if (psattn::bwd_scratch_bytes(meta, n_q_heads) > kStaticBytes) return PSATTN_ELIMIT;
    void* base = nullptr;
    const int rc = static_scratch(&base);
    if (rc != PSATTN_OK) return rc;
    // Nothing in the scratch has to start from zero: the dQ pass writes delta and the rescaled
    // LSE of every real (token, head) before the dK/dV pass reads them, and what earlier calls
    // left at padding positions is removed by the pair masks.
    return psattn::bwd_checked(meta, dt, n_q_heads, n_kv_heads, head_dim, scale, Q, K, V, O, dO, LSE, dQ, dK, dV,
                               base, kStaticBytes, hip_stream);
}

}  // extern "C"
