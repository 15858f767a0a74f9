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
//    padding.  Tiles are copied global -> LDS asynchronously, one tile ahead, into
//    the buffer the previous tile has just vacated; one barrier per tile.
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

// Mask arithmetic of PARTIAL tiles.  A lane's 32 score elements of a 64-row tile are
// numbered e = 16 b + i (b = 32-row block, i = accumulator register); element e belongs to
// tile row 32 b + acc_row(i, g), so the elements ordered by e are also ordered by row.
// elems_below(x, g): how many of them lie in rows below x, 0 <= x <= 64.
__device__ inline int elems_below(int x, int g) {
    return 4 * (x >> 3) + min(max((x & 7) - 4 * g, 0), 4);
}

// bit e set <=> element e lies in tile rows [lo, hi) (any integers; clamped to the tile)
__device__ inline uint32_t elem_range_bits(int lo, int hi, int g) {
    const int a = elems_below(min(max(lo, 0), 64), g), b = elems_below(min(max(hi, 0), 64), g);
    return static_cast<uint32_t>(((1ull << b) - 1) & ~((1ull << a) - 1));
}

// x if bit e of `bits` is set, otherwise -inf (two instructions: bit -> word mask, select)
template <int E>
__device__ __forceinline__ float keep_or_neg_inf(float x, uint32_t bits) {
    const uint32_t m = static_cast<uint32_t>(static_cast<int32_t>(bits << (31 - E)) >> 31);
    return __uint_as_float((__float_as_uint(x) & m) | (~m & 0xff800000u));
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

// Asynchronous global -> LDS copies (global_load_lds_*): no staging registers.
// One wave instruction writes lane l's 16 (or 4) bytes at LDS base + 16 (4) * l, the
// base being wave-uniform (M0).  The copies are issued from inline assembly on
// purpose: the compiler's wait-count bookkeeping treats every LDS read that follows a
// copy it knows of as dependent on it and waits for vmcnt(0) there, which would
// serialise each copy with the arithmetic it is meant to overlap.  Completion is
// therefore tracked by hand: copies retire in issue order, dma_wait_barrier<N>()
// waits until at most N of this wave's copies are in flight and then joins the
// workgroup barrier.  Compiler-issued vector memory loads stay correct (its waits can
// only be stricter than needed); inside the tile loops there are none except the tile
// list refills, which are consumed right after a full wait.
// The copies also write M0 (the LDS base).  The compiler refuses M0 in a clobber list (it is
// a reserved register), so the statements cannot declare it; what makes this sound is that
// compiled code for gfx950 keeps nothing alive in M0 in these kernels, which a test on the
// compiled ISA pins (no instruction outside the assembly statements names M0).
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) char*)p));
}

__device__ __forceinline__ void dma4(const void* src, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(src) : "memory");
}

template <int N>
__device__ __forceinline__ void dma_wait_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Copy of a 64-row tile (256-byte rows, rows `row_bytes` apart in global memory) into a
// swizzled LDS tile.  A wave instruction fills four tile rows, so the swizzle is applied
// on the global side: lane l fetches the logical chunk that belongs at physical chunk
// l % 16 of row r4 + l / 16.  Each of the four waves of a workgroup copies 16 rows in 4
// instructions; DmaLane holds the lane's byte offsets for them, so that a copy costs no
// vector ALU work: the address is a scalar tile base plus that 32-bit lane offset.
struct DmaLane {
    uint32_t off[4];
};

// `w` (wave index in the workgroup) must be wave-uniform; rows past `last_row` re-read it
__device__ __forceinline__ DmaLane dma_lane(uint32_t row_bytes, int w, int l, int last_row = 63) {
    DmaLane d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 16 * w + 4 * i + (l >> 4);
        const int sw = ((row & 3) << 2) | ((row >> 2) & 3);
        d.off[i] = static_cast<uint32_t>(min(row, last_row)) * row_bytes + (((l & 15) ^ sw) << 4);
    }
    return d;
}

__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(lane_off), "s"(base) : "memory");
}

// `base`: first row of the tile (wave-uniform); `tile`: LDS tile; `full`: the lane offsets
// of an unclipped tile; a tile whose last valid row is < 63 takes the clamped offsets.
__device__ __forceinline__ void dma_tile64(const char* base, uint32_t row_bytes, int last_row, const DmaLane& full, const char* tile, int w, int l) {
    const uint32_t lds = lds_addr(tile) + 16 * w * kRowBytes;
    if (last_row >= 63) {
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16(base, full.off[i], lds + 4 * i * kRowBytes);
    } else {
        asm volatile("; clipped tile" : "+s"(last_row));  // keeps the clamped offsets' arithmetic in this branch
        const DmaLane c = dma_lane(row_bytes, w, l, last_row);
#pragma unroll
        for (int i = 0; i < 4; ++i) dma16(base, c.off[i], lds + 4 * i * kRowBytes);
    }
}

// Copy of a pair of tiles (K and V of one key block, or Q and dO of one query block) as
// eight separate instructions per lane, so that a kernel can spread them over its MFMA
// slots: issued back to back they hold the wave for about a thousand cycles (the CU's
// address unit takes one such instruction per ~16 cycles and the waves of a workgroup issue
// theirs at the same moment).  One piece every other slot keeps the unit's queue short.
// Pieces 0-3 belong to the first tile, 4-7 to the second.
struct PairCopy {
    const char* a;  // first row of the first tile (wave-uniform)
    const char* b;  // first row of the second tile
    DmaLane lane;
};

__device__ __forceinline__ void pair_copy_setup(PairCopy& c, const char* a, const char* b, uint32_t row_bytes, int last_row,
                                                const DmaLane& full, int w, int l) {
    c.a = a;
    c.b = b;
    c.lane = full;
    if (last_row < 63) {
        asm volatile("; clipped tile" : "+s"(last_row));  // keeps the clamped offsets' arithmetic in this branch
        c.lane = dma_lane(row_bytes, w, l, last_row);
    }
}

template <int P>
__device__ __forceinline__ void pair_copy_piece(const PairCopy& c, const char* tile_a, const char* tile_b, int w) {
    if constexpr (P < 4) dma16(c.a, c.lane.off[P], lds_addr(tile_a) + (16 * w + 4 * P) * kRowBytes);
    else dma16(c.b, c.lane.off[P - 4], lds_addr(tile_b) + (16 * w + 4 * (P - 4)) * kRowBytes);
}

// Reader of a tile list walked in one direction: position k = 0, 1, ... maps to
// list[first + step * k] (step = +1 or -1), n positions in all.  Lane l keeps entry
// 64 b + l of the current batch b; the next batch is requested when a batch is entered,
// i.e. 64 positions before its first use.  get(k) must be called with non-decreasing k,
// from wave-uniform control flow, at a point where no asynchronous copy is in flight
// (the refill is a compiler-tracked load and is waited for with vmcnt(0)).
struct EntryStream {
    const int* list;
    int first, step, n, l;
    int cur, nxt, batch;
    __device__ __forceinline__ int fetch(int b) const {
        const int k = min(64 * b + l, n - 1);
        return list[first + step * k];
    }
    __device__ __forceinline__ void init(const int* list_, int first_, int step_, int n_, int l_) {
        list = list_; first = first_; step = step_; n = n_; l = l_;
        batch = 0;
        cur = n > 0 ? fetch(0) : 0;
        nxt = n > 64 ? fetch(1) : 0;
    }
    __device__ __forceinline__ int get(int k) {
        if ((k >> 6) != batch) {
            batch = k >> 6;
            cur = nxt;
            if (64 * (batch + 1) < n) nxt = fetch(batch + 1);
        }
        return __builtin_amdgcn_readlane(cur, k & 63);
    }
};

// ---- rotary position embedding (Section 3.1: position ids follow the paired format)
// Dimension i < 64 is paired with i + 64 and the pair is turned by the angle of (position, i).
// The table row of a position holds cos of the 64 angles, then sin.  All layouts in these kernels
// keep both members of a pair in the same lane, so rotating is lane-local.

// position id of token t: prompt and first response count on from the sample's start; a later
// response skips the hidden range [hole_lo, hole_hi), which puts it right behind the prompt
__device__ inline int rope_position(const Tok4& tk, int t) {
    return tk.s == kPadStart ? 0 : t - tk.s - (tk.hole_hi - tk.hole_lo);
}

// (x1, x2) -> turned by +angle (inverse = false) or -angle (inverse = true)
template <bool INVERSE>
__device__ __forceinline__ void rope_turn(float& x1, float& x2, float c, float s) {
    const float y1 = INVERSE ? fmaf(x2, s, x1 * c) : fmaf(-x2, s, x1 * c);
    const float y2 = INVERSE ? fmaf(-x1, s, x2 * c) : fmaf(x1, s, x2 * c);
    x1 = y1;
    x2 = y2;
}

// Rotates 8 packed bf16 (dims i0 .. i0 + 7, i0 < 64) and their partners (dims 64 + i0 ..) in place;
// `row` points at the table row of the token's position.
__device__ inline void rope_frag8(Frag8& lo, Frag8& hi, const float* row, int i0) {
    const float4 c0 = *reinterpret_cast<const float4*>(row + i0), c1 = *reinterpret_cast<const float4*>(row + i0 + 4);
    const float4 s0 = *reinterpret_cast<const float4*>(row + 64 + i0), s1 = *reinterpret_cast<const float4*>(row + 64 + i0 + 4);
    const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    uint32_t lw[4] = {lo.u.x, lo.u.y, lo.u.z, lo.u.w}, hw[4] = {hi.u.x, hi.u.y, hi.u.z, hi.u.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float a0 = __uint_as_float(lw[j] << 16), a1 = __uint_as_float(lw[j] & 0xffff0000u);
        float b0 = __uint_as_float(hw[j] << 16), b1 = __uint_as_float(hw[j] & 0xffff0000u);
        rope_turn<false>(a0, b0, cs[2 * j], sn[2 * j]);
        rope_turn<false>(a1, b1, cs[2 * j + 1], sn[2 * j + 1]);
        f32x2 va = {a0, a1}, vb = {b0, b1};
        lo.p[j] = __builtin_convertvector(va, bf16x2);
        hi.p[j] = __builtin_convertvector(vb, bf16x2);
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
