// bf16 flash-attention kernels for gfx950 (MI355X), head_dim 128.
//
// What is computed is ordinary softmax attention on the pairs allowed by the
// prefix-sharing mask (paper Algorithm 1 / Algorithm 3); tiles of the block mask
// without an allowed pair are never visited (Section 3.1).  How it is computed is
// this file's own design:
//
//  * 64-wide wavefronts, v_mfma_f32_32x32x16_bf16.  Every product is arranged so
//    that the quantity the wave owns (its 32 queries in forward / dQ, its 32 keys
//    in dK/dV) is the MFMA *column*: scores come out with one query (or key) per
//    lane, softmax statistics are per-lane scalars, and the probabilities feed the
//    next MFMA as a B operand straight from the accumulator registers (the
//    accumulator's row order is absorbed into the order in which the other
//    operand's rows are fetched).
//  * K/V (or Q/dO) tiles are staged in LDS, 256-byte rows, with the 16-byte chunk
//    index XOR-swizzled by the row so that both row-wise 128-bit reads and the
//    transposing 64-bit reads (ds_read_b64_tr_b16) are bank-conflict free without
//    padding.  The next tile's global loads are issued before the current tile's
//    math and parked in registers.
//  * dK/dV are owned by one workgroup per (k-tile, kv-head), which walks the G
//    query heads of the group and the k-major tile list, so the prompt's keys
//    collect the contributions of prompt, chosen and rejected queries without
//    atomics.  dQ is a separate q-major pass.  Both are deterministic.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "psattn_internal.h"

namespace psattn {
namespace mma {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kRowBytes = 256;  // 128 bf16

// compile-time loop: f(std::integral_constant<int, I>) for I in [B, E)
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

union Frag8 {
    bf16x8 v;
    bf16x4 h[2];
    bf16x2 p[4];
    uint4 u;
};

// byte offset of 16-byte chunk `chunk` of row `row` in a swizzled tile
__device__ inline int tile_off(int row, int chunk) {
    const int sw = ((row & 3) << 2) | ((row >> 2) & 3);
    return row * kRowBytes + ((chunk ^ sw) << 4);
}

// MFMA A operand, rows taken as they are stored: 8 consecutive bf16 of one row.
__device__ inline bf16x8 lds_rows(const char* tile, int row, int chunk) {
    return *reinterpret_cast<const bf16x8*>(tile + tile_off(row, chunk));
}

// MFMA A operand of the transposed tile: lane (l % 32) is column col0 + l % 32 of
// the stored tile, its 8 values are stored rows r0 + {0..3} and r0 + 8 + {0..3}
// where r0 = row0 + 4 * (l / 32).  This is the row order in which a 32x32
// accumulator hands its values to the next MFMA.
__device__ inline bf16x8 lds_cols(const char* tile, int row0, int col0, int l) {
    const int i16 = l & 15;
    const int row = row0 + 4 * (l >> 5) + (i16 >> 2);
    const int col = col0 + 16 * ((l >> 4) & 1) + 4 * (i16 & 3);
    const int sub = (col & 7) * 2;
    Frag8 f;
    f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (lds_bf16x4*)(tile + tile_off(row, col >> 3) + sub));
    f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        (lds_bf16x4*)(tile + tile_off(row + 8, col >> 3) + sub));
    return f.v;
}

// Per-lane LDS byte offsets of the two operand fetch patterns, relative to the first
// row of a 32-row block.  Because the swizzle is an XOR on the 16-byte chunk index,
// the offset for step t (row-wise operand) or head-dim block db (transposed operand)
// is one lane constant XOR a compile-time constant:
//   row-wise, step t:        nat ^ (t << 5)     row l % 32, chunk 2 t + l / 32
//   transposed, block db:    tr1 ^ (db << 6)    rows 4 (l / 32) + (l % 16) / 4, first four
//                            tr2 ^ (db << 6)    the same, eight rows further down
// A tile base that is a multiple of 256 bytes may be added to the lane constant first.
struct LaneOffsets {
    int nat, tr1, tr2;
};

__device__ inline LaneOffsets lane_offsets(int l) {
    LaneOffsets o;
    const int c32 = l & 31, g = l >> 5, i16 = l & 15;
    o.nat = tile_off(c32, g);
    const int row = 4 * g + (i16 >> 2);
    const int col = 16 * ((l >> 4) & 1) + 4 * (i16 & 3);
    o.tr1 = tile_off(row, col >> 3) + (col & 7) * 2;
    o.tr2 = tile_off(row + 8, col >> 3) + (col & 7) * 2;
    return o;
}

// row-wise MFMA operand, step t, of the 32-row block at `blk` (blk: multiple of 256 bytes)
template <int T>
__device__ __forceinline__ bf16x8 ld_rows(const char* blk, int nat) {
    return *reinterpret_cast<const bf16x8*>(blk + (nat ^ (T << 5)));
}

// transposed MFMA operand: head-dim block DB, stored rows 16 HALF + {0..15} of the block
template <int DB, int HALF>
__device__ __forceinline__ bf16x8 ld_cols(const char* blk, int tr1, int tr2) {
    Frag8 f;
    f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(blk + (tr1 ^ (DB << 6)) + 16 * HALF * kRowBytes));
    f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(blk + (tr2 ^ (DB << 6)) + 16 * HALF * kRowBytes));
    return f.v;
}

__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// values of accumulator registers [8*half, 8*half + 8) as a bf16 B operand
__device__ inline bf16x8 pack8(const f32x16& x, int half) {
    Frag8 f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x2 v = {x[8 * half + 2 * j], x[8 * half + 2 * j + 1]};
        f.p[j] = __builtin_convertvector(v, bf16x2);
    }
    return f.v;
}

// max / sum across the two half-waves that share a column
__device__ inline float other_half(float x) {
    const uint32_t u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(threadIdx.x & 32 ? r[0] : r[1]);
}

// row of the 32x32 accumulator that register i of lane-half g holds
__device__ inline int acc_row(int i, int g) { return (i >> 2) * 8 + 4 * g + (i & 3); }

// Asynchronous copy of a 64-row x 256-byte tile from global memory straight into a
// swizzled LDS tile (global_load_lds_dwordx4: no staging registers, no ds_write).
// A wave instruction writes 64 x 16 bytes to consecutive LDS addresses in lane order
// = four tile rows, so the swizzle is applied on the global side: lane l fetches the
// logical chunk that belongs at physical chunk l % 16 of row r4 + l / 16.  Each of the
// four waves of a workgroup copies 16 rows.  `base` points at row `row0` ... the tile's
// rows are `row_bytes` apart; rows past `last_row` (relative to row0) re-read that row.
// Completion is tracked by vmcnt; __syncthreads() waits for it.
__device__ __forceinline__ void dma_tile64(const char* base, uint32_t row_bytes, int last_row, char* tile, int w, int l) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r4 = 16 * w + 4 * i;
        const int row = r4 + (l >> 4);
        const int sw = ((row & 3) << 2) | ((row >> 2) & 3);
        const char* src = base + static_cast<uint32_t>(min(row, last_row)) * row_bytes + (((l & 15) ^ sw) << 4);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(tile + r4 * kRowBytes), 16, 0, 0);
    }
}

struct Stage {  // one thread's share of a 64 x 128 bf16 tile: 4 chunks of 16 bytes
    u32x4 c[4];
};

__device__ inline void stage_load(Stage& s, const uint16_t* base, int row0, int T, size_t row_stride,
                                  int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
        const int tok = row0 + row;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        s.c[i] = tok < T ? *reinterpret_cast<const u32x4*>(base + static_cast<size_t>(tok) * row_stride + ch * 8)
                         : zero;
    }
}

// Same, but rows past the end of the buffer re-read the last token (no branch); the
// caller masks whatever those rows produce.
__device__ inline void stage_load_clamped(Stage& s, const uint16_t* base, int row0, int T, size_t row_stride,
                                          int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
        const int tok = min(row0 + row, T - 1);
        s.c[i] = *reinterpret_cast<const u32x4*>(base + static_cast<size_t>(tok) * row_stride + ch * 8);
    }
}

__device__ inline void stage_store(const Stage& s, char* tile, int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
        *reinterpret_cast<u32x4*>(tile + tile_off(row, ch)) = s.c[i];
    }
}

__device__ inline void store4(uint16_t* dst, float a, float b, float c, float d) {
    f32x2 v0 = {a, b}, v1 = {c, d};
    union { bf16x2 p[2]; uint2 u; } o;
    o.p[0] = __builtin_convertvector(v0, bf16x2);
    o.p[1] = __builtin_convertvector(v1, bf16x2);
    *reinterpret_cast<uint2*>(dst) = o.u;
}

}  // namespace mma
}  // namespace psattn
