// Plain-FMA kernels for any tile grid, float or bfloat16 storage, head_dim 64 or
// 128.  They serve the fp32 configuration (where the 1e-5 tolerance rules out
// bf16 matrix cores) and every shape the MFMA kernels are not built for.  One
// thread owns one query row (forward, dQ) or one key row (dK/dV); scores are
// never stored.  All accumulation is fp32 with expf/logf.
//
// The tile lists come from the block mask (paper Section 3.1): only tiles that
// hold an allowed pair are visited, FULL tiles skip the per-pair mask test of
// Algorithm 3.
#include <hip/hip_runtime.h>

#include "psattn_internal.h"

namespace psattn {
namespace {

__device__ inline float ld(const float* p) { return *p; }
__device__ inline float ld(const uint16_t* p) { return __uint_as_float(static_cast<uint32_t>(*p) << 16); }
__device__ inline void st(float* p, float v) { *p = v; }
__device__ inline void st(uint16_t* p, float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) { *p = static_cast<uint16_t>((u >> 16) | 0x40); return; }
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = static_cast<uint16_t>(u >> 16);
}

__device__ inline bool allowed(const Tok4& t, int q, int kv) {
    return kv >= t.s && kv <= q && !(kv >= t.hole_lo && kv < t.hole_hi);
}

constexpr int kThreads = 64;

// ---------------------------------------------------------------- forward
template <typename E, int D>
__global__ __launch_bounds__(kThreads) void generic_fwd(AttnArgs a) {
    const DeviceCsr& g = a.meta.fwd;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv;
    const int tile = g.order[blockIdx.x / Hq];
    const int h = blockIdx.x % Hq, kvh = h / (Hq / Hkv);
    const E* Q = static_cast<const E*>(a.Q);
    const E* K = static_cast<const E*>(a.K);
    const E* V = static_cast<const E*>(a.V);
    E* O = static_cast<E*>(a.Oout);
    const int q_end = min(T, (tile + 1) * g.tile_q);
    for (int i = tile * g.tile_q + threadIdx.x; i < q_end; i += kThreads) {
        const Tok4 t = a.meta.tok[i];
        float q[D], acc[D];
#pragma unroll
        for (int x = 0; x < D; ++x) { q[x] = ld(Q + (static_cast<size_t>(i) * Hq + h) * D + x); acc[x] = 0.f; }
        float m = -INFINITY, l = 0.f;
        for (int e = g.row_ptr[tile]; e < g.row_ptr[tile + 1]; ++e) {
            const int ent = g.entry[e];
            const int k0 = (ent >> 2) * g.tile_k, k1 = min(T, k0 + g.tile_k);
            const bool full = (ent & 3) == PSATTN_TILE_FULL;
            for (int j = k0; j < k1; ++j) {
                if (!full && !allowed(t, i, j)) continue;
                const E* kr = K + (static_cast<size_t>(j) * Hkv + kvh) * D;
                const E* vr = V + (static_cast<size_t>(j) * Hkv + kvh) * D;
                float s = 0.f;
#pragma unroll
                for (int x = 0; x < D; ++x) s = fmaf(q[x], ld(kr + x), s);
                s *= a.scale;
                const float mn = fmaxf(m, s);
                const float alpha = expf(m - mn);  // m = -inf the first time: 0
                const float p = expf(s - mn);
                l = l * alpha + p;
#pragma unroll
                for (int x = 0; x < D; ++x) acc[x] = fmaf(p, ld(vr + x), acc[x] * alpha);
                m = mn;
            }
        }
        const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
        for (int x = 0; x < D; ++x) st(O + (static_cast<size_t>(i) * Hq + h) * D + x, acc[x] * inv);
        a.LSEout[static_cast<size_t>(h) * T + i] = l > 0.f ? m + logf(l) : -INFINITY;
    }
}

// ---------------------------------------------------------------- delta = rowsum(dO o O)
template <typename E>
__global__ __launch_bounds__(256) void delta_kernel(AttnArgs a) {
    const int T = a.meta.T, Hq = a.Hq, D = a.d;
    const int lanes = 16;  // threads per (token, head) row
    const size_t row = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) / lanes;
    const int sub = threadIdx.x % lanes;
    const size_t n_rows = static_cast<size_t>(T) * Hq;
    float s = 0.f;
    if (row < n_rows) {
        const E* o = static_cast<const E*>(a.O) + row * D;
        const E* g = static_cast<const E*>(a.dO) + row * D;
        for (int x = sub; x < D; x += lanes) s = fmaf(ld(o + x), ld(g + x), s);
    }
#pragma unroll
    for (int off = lanes / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (row < n_rows && sub == 0) {
        const size_t t = row / Hq, h = row % Hq;
        a.delta[h * T + t] = s;
    }
}

// ---------------------------------------------------------------- dQ (q-major)
template <typename E, int D>
__global__ __launch_bounds__(kThreads) void generic_dq(AttnArgs a) {
    const DeviceCsr& g = a.meta.fwd;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv;
    const int tile = g.order[blockIdx.x / Hq];
    const int h = blockIdx.x % Hq, kvh = h / (Hq / Hkv);
    const E* Q = static_cast<const E*>(a.Q);
    const E* K = static_cast<const E*>(a.K);
    const E* V = static_cast<const E*>(a.V);
    const E* dO = static_cast<const E*>(a.dO);
    E* dQ = static_cast<E*>(a.dQ);
    const int q_end = min(T, (tile + 1) * g.tile_q);
    for (int i = tile * g.tile_q + threadIdx.x; i < q_end; i += kThreads) {
        const Tok4 t = a.meta.tok[i];
        float q[D], go[D], acc[D];
#pragma unroll
        for (int x = 0; x < D; ++x) {
            q[x] = ld(Q + (static_cast<size_t>(i) * Hq + h) * D + x);
            go[x] = ld(dO + (static_cast<size_t>(i) * Hq + h) * D + x);
            acc[x] = 0.f;
        }
        const float lse = a.LSE[static_cast<size_t>(h) * T + i];
        const float dl = a.delta[static_cast<size_t>(h) * T + i];
        for (int e = g.row_ptr[tile]; e < g.row_ptr[tile + 1]; ++e) {
            const int ent = g.entry[e];
            const int k0 = (ent >> 2) * g.tile_k, k1 = min(T, k0 + g.tile_k);
            const bool full = (ent & 3) == PSATTN_TILE_FULL;
            for (int j = k0; j < k1; ++j) {
                if (!full && !allowed(t, i, j)) continue;
                const E* kr = K + (static_cast<size_t>(j) * Hkv + kvh) * D;
                const E* vr = V + (static_cast<size_t>(j) * Hkv + kvh) * D;
                float s = 0.f, dp = 0.f;
#pragma unroll
                for (int x = 0; x < D; ++x) { s = fmaf(q[x], ld(kr + x), s); dp = fmaf(go[x], ld(vr + x), dp); }
                const float p = expf(s * a.scale - lse);
                const float ds = p * (dp - dl);
#pragma unroll
                for (int x = 0; x < D; ++x) acc[x] = fmaf(ds, ld(kr + x), acc[x]);
            }
        }
#pragma unroll
        for (int x = 0; x < D; ++x) st(dQ + (static_cast<size_t>(i) * Hq + h) * D + x, acc[x] * a.scale);
    }
}

// ---------------------------------------------------------------- dK, dV (k-major)
template <typename E, int D>
__global__ __launch_bounds__(kThreads) void generic_dkdv(AttnArgs a) {
    const DeviceCsr& g = a.meta.bwd;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const int tile = g.order[blockIdx.x / Hkv];
    const int kvh = blockIdx.x % Hkv;
    const E* Q = static_cast<const E*>(a.Q);
    const E* K = static_cast<const E*>(a.K);
    const E* V = static_cast<const E*>(a.V);
    const E* dO = static_cast<const E*>(a.dO);
    E* dK = static_cast<E*>(a.dK);
    E* dV = static_cast<E*>(a.dV);
    const int k_end = min(T, (tile + 1) * g.tile_k);
    for (int j = tile * g.tile_k + threadIdx.x; j < k_end; j += kThreads) {
        const int q_hi = a.meta.tok[j].key_hi;  // queries [j, q_hi) may read key j
        float dk[D], dv[D];
#pragma unroll
        for (int x = 0; x < D; ++x) { dk[x] = 0.f; dv[x] = 0.f; }
        const E* kr = K + (static_cast<size_t>(j) * Hkv + kvh) * D;
        const E* vr = V + (static_cast<size_t>(j) * Hkv + kvh) * D;
        for (int gi = 0; gi < G; ++gi) {
            const int h = kvh * G + gi;
            for (int e = g.row_ptr[tile]; e < g.row_ptr[tile + 1]; ++e) {
                const int ent = g.entry[e];
                const int q0 = (ent >> 2) * g.tile_q, q1 = min(T, q0 + g.tile_q);
                for (int i = max(q0, j); i < min(q1, q_hi); ++i) {
                    const E* qr = Q + (static_cast<size_t>(i) * Hq + h) * D;
                    const E* gr = dO + (static_cast<size_t>(i) * Hq + h) * D;
                    float s = 0.f, dp = 0.f;
#pragma unroll
                    for (int x = 0; x < D; ++x) { s = fmaf(ld(qr + x), ld(kr + x), s); dp = fmaf(ld(gr + x), ld(vr + x), dp); }
                    const float p = expf(s * a.scale - a.LSE[static_cast<size_t>(h) * T + i]);
                    const float ds = p * (dp - a.delta[static_cast<size_t>(h) * T + i]);
#pragma unroll
                    for (int x = 0; x < D; ++x) { dv[x] = fmaf(p, ld(gr + x), dv[x]); dk[x] = fmaf(ds, ld(qr + x), dk[x]); }
                }
            }
        }
#pragma unroll
        for (int x = 0; x < D; ++x) {
            st(dK + (static_cast<size_t>(j) * Hkv + kvh) * D + x, dk[x] * a.scale);
            st(dV + (static_cast<size_t>(j) * Hkv + kvh) * D + x, dv[x]);
        }
    }
}

hipError_t last_error() { return hipGetLastError(); }

}  // namespace

#define PSATTN_DISPATCH(KERNEL, GRID)                                                              \
    do {                                                                                           \
        hipStream_t s = static_cast<hipStream_t>(stream);                                          \
        if (GRID == 0) return 0;                                                                   \
        if (dt == PSATTN_F32 && a.d == 64) KERNEL<float, 64><<<GRID, kThreads, 0, s>>>(a);         \
        else if (dt == PSATTN_F32 && a.d == 128) KERNEL<float, 128><<<GRID, kThreads, 0, s>>>(a);  \
        else if (dt == PSATTN_BF16 && a.d == 64) KERNEL<uint16_t, 64><<<GRID, kThreads, 0, s>>>(a);\
        else KERNEL<uint16_t, 128><<<GRID, kThreads, 0, s>>>(a);                                   \
        return static_cast<int>(last_error());                                                     \
    } while (0)

int launch_generic_fwd(int dt, const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    PSATTN_DISPATCH(generic_fwd, grid);
}
int launch_generic_dq(int dt, const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    PSATTN_DISPATCH(generic_dq, grid);
}
int launch_generic_dkdv(int dt, const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.bwd.n_rows) * a.Hkv;
    PSATTN_DISPATCH(generic_dkdv, grid);
}
int launch_delta(int dt, const AttnArgs& a, void* stream) {
    const size_t rows = static_cast<size_t>(a.meta.T) * a.Hq;
    const unsigned grid = static_cast<unsigned>((rows * 16 + 255) / 256);
    if (grid == 0) return 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == PSATTN_F32) delta_kernel<float><<<grid, 256, 0, s>>>(a);
    else delta_kernel<uint16_t><<<grid, 256, 0, s>>>(a);
    return static_cast<int>(last_error());
}

}  // namespace psattn
