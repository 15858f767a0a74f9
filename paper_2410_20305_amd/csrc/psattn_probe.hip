// Measurement aid for one design decision: should the backward be ONE k-major pass that
// also accumulates dQ with fp32 atomic adds, instead of the separate q-major dQ pass?
// This kernel issues exactly the memory operations such a pass would add, and nothing else:
// one workgroup per (k-tile, kv-head) walks the k-major tile list of the block mask and,
// for every (q-tile, q-head) it visits, adds a 64 x 128 fp32 tile into a [T, Hq, 128]
// accumulator.  Lanes are laid out as the 32x32 MFMA accumulator would hand the values
// over (wave w owns head dims 32 w .. 32 w + 31, one lane per head dim, 16 query rows per
// lane and 32-query block), so each wave instruction covers two full 128-byte lines: the
// most coalesced form this access pattern has.  mode 0: atomic adds; mode 1: plain stores
// of the same addresses (what a write-partials-then-reduce scheme would cost at least).
#include <hip/hip_runtime.h>

#include "psattn_internal.h"

namespace psattn {
namespace {

__global__ __launch_bounds__(256) void psattn_dq_atomics_probe(DeviceMeta meta, int Hq, int Hkv, float* acc, int mode) {
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, g = l >> 5;
    const int G = Hq / Hkv, T = meta.T;
    const DeviceCsr& csr = meta.bwd;
    const RowLaunch rl = csr.launch[blockIdx.x / Hkv];
    const int kvh = blockIdx.x % Hkv;
    for (int k = rl.count - 1; k >= 0; --k) {  // same walk as the dK/dV kernel: last q-tile first, heads innermost
        const int q0 = (csr.entry[rl.begin + k] >> 2) * csr.tile_q;
        for (int hh = 0; hh < G; ++hh) {
            const int h = kvh * G + hh;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int q = min(q0 + 32 * b + (i >> 2) * 8 + 4 * g + (i & 3), T - 1);
                    float* p = acc + (static_cast<size_t>(q) * Hq + h) * 128 + 32 * w + c32;
                    if (mode == 0) unsafeAtomicAdd(p, 1.0f);
                    else __builtin_nontemporal_store(1.0f, p);
                }
        }
    }
}

// What the matrix cores sustain when nothing else issues: every wave runs `iters` rounds of four
// independent v_mfma_f32_32x32x16_bf16 chains on register operands (no memory traffic at all).
// With the clock the device holds under this load it is the ceiling any MFMA-bound kernel has.
// MODE 0: one constant fragment per operand side (the data paths hardly toggle).
// MODE 1: eight different fragments per side holding pseudo-random values (random sign and mantissa,
// magnitudes 0.5 to 2), a different pair on every MFMA: the clock the device holds depends on the data.
// MODE 2: the register pattern of mode 1 with the constant values of mode 0 (tells the data apart
// from the operand registers changing on every MFMA).
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 probe_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_f32x16;

// Two bf16 values in one register: random sign and mantissa, exponent 126 or 127 (magnitudes 0.5 to 2, zero mean)
__device__ inline uint32_t probe_pair(uint32_t key) {
    key = key * 1664525u + 1013904223u;
    key ^= key >> 15;
    key *= 2246822519u;
    key ^= key >> 13;
    return 0x3F003F00u | (key & 0x80FF80FFu);
}

template <int MODE>
__global__ __launch_bounds__(256) void psattn_mfma_peak_probe(int iters, float* sink) {
    constexpr int F = MODE ? 8 : 1;
    constexpr bool RANDOM = MODE == 1;
    union Frag { probe_bf16x8 v; uint32_t u[4]; };
    Frag fa[F], fb[F];
    probe_bf16x8 a[F], b[F];
    const uint32_t lane_key = (blockIdx.x * 256u + threadIdx.x) * 64u;
#pragma unroll
    for (int f = 0; f < F; ++f) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            fa[f].u[j] = RANDOM ? probe_pair(lane_key + 8 * f + 2 * j) : 0x3F803F80u;      // constant: 1.0
            fb[f].u[j] = RANDOM ? probe_pair(lane_key + 8 * f + 2 * j + 1) : 0x3F003F00u;  // constant: 0.5
        }
        a[f] = fa[f].v;
        b[f] = fb[f].v;
        asm volatile("" : "+v"(a[f]), "+v"(b[f]));  // every fragment in registers of its own
    }
    probe_f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; i += 2) {  // eight MFMAs per turn; `iters` is even
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1 % F], b[1 % F], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 % F], b[2 % F], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3 % F], b[3 % F], c3, 0, 0, 0);
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[4 % F], b[4 % F], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[5 % F], b[5 % F], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[6 % F], b[6 % F], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[7 % F], b[7 % F], c3, 0, 0, 0);
    }
    float r = 0.f;
    for (int j = 0; j < 16; ++j) r += c0[j] + c1[j] + c2[j] + c3[j];
    if (r == 12345.678f) sink[0] = r;  // keeps the chains alive; never true
}

}  // namespace
}  // namespace psattn

extern "C" int psattn_probe_mfma_peak(int32_t n_workgroups, int32_t iters, int32_t random_operands, float* sink,
                                      void* hip_stream) {
    if (n_workgroups <= 0 || iters <= 0 || (iters & 1) || random_operands < 0 || random_operands > 2 || !sink) return PSATTN_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (random_operands == 1) psattn::psattn_mfma_peak_probe<1><<<n_workgroups, 256, 0, st>>>(iters, sink);
    else if (random_operands == 2) psattn::psattn_mfma_peak_probe<2><<<n_workgroups, 256, 0, st>>>(iters, sink);
    else psattn::psattn_mfma_peak_probe<0><<<n_workgroups, 256, 0, st>>>(iters, sink);
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}

extern "C" int psattn_probe_dq_atomics(const psattn_meta* meta, int32_t n_q_heads, int32_t n_kv_heads, float* acc,
                                       int32_t mode, void* hip_stream) {
    if (!meta || !acc || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0) return PSATTN_EINVAL;
    if (!meta->on_device) return PSATTN_ENODEVICE;
    if (meta->bwd.tile_q != psattn::kBwdTileQ || meta->bwd.tile_k != psattn::kBwdTileK) return PSATTN_EUNSUPPORTED;
    const unsigned grid = static_cast<unsigned>(meta->dev.bwd.n_rows) * n_kv_heads;
    if (grid == 0) return PSATTN_OK;
    psattn::psattn_dq_atomics_probe<<<grid, 256, 0, static_cast<hipStream_t>(hip_stream)>>>(meta->dev, n_q_heads, n_kv_heads,
                                                                                           acc, mode);
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}
