// bf16 MFMA dK/dV kernel for gfx950; layout and staging helpers are in psattn_mfma_common.h.
//
// grid: one workgroup per (k-tile of 128 keys, kv-head); 4 waves x 32 keys, one wave per
// SIMD.  The workgroup walks the G query heads of its group and, for each, the q-tiles
// (64 queries) that can read its keys (the k-major tile list of the block mask, paper
// Section 3.1), so the prompt's keys collect the contributions of prompt, chosen and
// rejected queries in one place, without atomics.
//
// Register plan.  A wave keeps dK and dV of its 32 keys (2 x 64 fp32 per lane) and its K
// and V fragments (2 x 32 registers per lane) for the whole kernel: 192 registers that only
// MFMA instructions ever touch.  They live in the accumulation registers a[0:191], which
// MFMA reads and writes directly and the vector ALU cannot address; the ordinary registers
// are left to the scores, the LDS operand ring and the softmax arithmetic.  The compiler
// cannot express this split (once a kernel needs more than 256 registers it sends either
// every MFMA result or none to the accumulation registers, and moves whole accumulators
// back and forth), so all MFMAs of this kernel are issued from inline assembly that names
// the accumulation registers itself; everything else is ordinary compiled code.  This file
// is built with the compiler's own use of accumulation registers for spilling switched off,
// so a[0:191] belong to the assembly alone.
//
// The compiler does not know that the assembly statements are MFMAs and inserts no wait
// states after them: settle() stands wherever another kind of instruction reads what a
// chain of MFMAs has produced.
#include "psattn_mfma_common.h"

namespace psattn {
namespace {
using namespace mma;

constexpr int kAccDV = 0;     // a[16 db + i]: dV^T block db (head dims 32 db ..), accumulator element i
constexpr int kAccDK = 64;    // likewise dK^T
constexpr int kRegK = 128;    // a[128 + 4 t ..]: K fragment of step t (head dims 16 t ..), B operand
constexpr int kRegV = 160;    // likewise V
constexpr int kAccRegs = 192;

// a[A0 : A0 + 15] += x y
template <int A0>
__device__ __forceinline__ void acc_mfma(bf16x8 x, bf16x8 y) {
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%0:%1], %2, %3, a[%0:%1]" ::"n"(A0), "n"(A0 + 15), "v"(x), "v"(y));
}

// acc (ordinary registers) = x * a[B0 : B0 + 3] (+ acc unless FIRST)
template <int B0, bool FIRST>
__device__ __forceinline__ void score_mfma(f32x16& acc, bf16x8 x) {
    if constexpr (FIRST)
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], 0" : "=&v"(acc) : "v"(x), "n"(B0), "n"(B0 + 3));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[%2:%3], %0" : "+v"(acc) : "v"(x), "n"(B0), "n"(B0 + 3));
}

template <int A>
__device__ __forceinline__ void acc_set(uint32_t v) {
    asm volatile("v_accvgpr_write_b32 a[%0], %1" ::"n"(A), "v"(v));
}

template <int A>
__device__ __forceinline__ float acc_get() {
    float v;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(A));
    return v;
}

// 24 wait states: more than the longest MFMA needs before its result may be read
__device__ __forceinline__ void settle() {
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
}

// ------------------------------------------------------------------ one q-tile
// With one wave per SIMD nothing hides latency but the wave's own instruction stream, so a
// q-tile is processed as 64 explicitly ordered slots, one MFMA each:
//   slots  0-15  S, dP of queries 0-31
//   slots 16-31  S, dP of queries 32-63      + softmax/dS arithmetic of queries 0-31
//   slots 32-47  dV, dK from queries 0-31    + softmax/dS arithmetic of queries 32-63
//   slots 48-63  dV, dK from queries 32-63
// The LDS operand of slot m is requested kAhead slots earlier into a register ring.

constexpr int kQTileBytes = 64 * kRowBytes;
constexpr int kAhead = 4;  // measured: 3 and 5 are both slower

// AND-masks for the packed bf16 pairs (elements 2j, 2j + 1 of block b) of one q-tile:
// the queries allowed to read this lane's key are rows [lo, hi) of the tile.
__device__ inline void pair_masks(uint32_t (&mw)[2][8], int lo, int hi, int g) {
    const uint32_t bits = elem_range_bits(lo, hi, g);
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = 16 * b2 + 2 * j;
            mw[b2][j] = ((bits >> e) & 1u ? 0x0000ffffu : 0u) | ((bits >> (e + 1)) & 1u ? 0xffff0000u : 0u);
        }
}

__device__ inline uint32_t pack2(float a, float b) {
    f32x2 v = {a, b};
    union { bf16x2 p; uint32_t u; } o;
    o.p = __builtin_convertvector(v, bf16x2);
    return o.u;
}

__device__ inline float comp(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// The LDS operands of the first kAhead slots (Q and dO rows of query block 0, head dims 0-31),
// requested as soon as the tile's data is visible so that the list bookkeeping between the barrier
// and the first MFMA overlaps their latency (configuration 5: 8.38 -> 8.30 ms).
__device__ __forceinline__ void tile_prefetch(Frag8 (&ring)[8], const char* sQ, const char* sG, const LaneOffsets& lo) {
    static_for<0, kAhead>([&](auto M) {
        constexpr int m = decltype(M)::value, t = m >> 1;
        ring[m & 7].v = ld_rows<t>((m & 1) ? sG : sQ, lo.nat);
    });
}

// FULL: every pair of the tile is allowed, no mask work at all (mw is not read).
// copy_piece(k), k = 0 .. 8, issues one instruction of the next tile's asynchronous copy;
// the pieces are spread over the first slots.
template <bool FULL, typename CopyPiece>
__device__ __forceinline__ void dkdv_tile(const char* sQ, const char* sG, const float* sL, const float* sD,
                                          const LaneOffsets& lo, const uint32_t (&mw)[2][8], float c, int g,
                                          Frag8 (&ring)[8], CopyPiece&& copy_piece) {
    f32x16 s[2], dp[2];
    u32x4 pw[2][2], dw[2][2];  // packed P and dS of a block: [block][half] is one B operand
    float4 Lc, Ln;
    float p0 = 0.f, p1 = 0.f;

    auto request = [&](auto M) {  // LDS operand of slot m -> ring[m % 8]
        constexpr int m = decltype(M)::value;
        if constexpr (m < 32) {
            constexpr int b = m >> 4, t = (m & 15) >> 1;
            const char* x = (m & 1) ? sG : sQ;
            ring[m & 7].v = ld_rows<t>(x + b * 32 * kRowBytes, lo.nat);
        } else if constexpr (m < 64) {
            constexpr int j = (m - 32) & 15, b = (m - 32) >> 4, half = j >> 3, db = (j & 7) >> 1;
            const char* x = (j & 1) ? sQ : sG;
            ring[m & 7].v = ld_cols<db, half>(x + 32 * b * kRowBytes, lo.tr1, lo.tr2);
        }
    };
    // dP accumulators of block b start from -delta of their queries (element i belongs to
    // query 32 b + acc_row(i, g)), so that dS = P o (dP - delta) is one multiplication
    auto start_dp = [&](auto B) {
        constexpr int b = decltype(B)::value;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const float4 d = *reinterpret_cast<const float4*>(sD + 32 * b + 8 * i4 + 4 * g);
            dp[b][4 * i4] = d.x; dp[b][4 * i4 + 1] = d.y; dp[b][4 * i4 + 2] = d.z; dp[b][4 * i4 + 3] = d.w;
        }
    };
    auto lse4 = [&](int b, int i4) {  // LSE * log2 e of 4 consecutive queries
        return *reinterpret_cast<const float4*>(sL + 32 * b + 8 * i4 + 4 * g);
    };

    // slots 0 .. kAhead - 1 were requested by the caller right behind the barrier (tile_prefetch)
    start_dp(std::integral_constant<int, 0>{});
    Lc = lse4(0, 0);
    static_for<0, 64>([&](auto M) {
        constexpr int m = decltype(M)::value;
        request(std::integral_constant<int, m + kAhead>{});
        // Copy pieces go out every other slot: the four waves issue theirs at the same moment and
        // the CU's address unit takes one such instruction per ~16 cycles, so a piece per slot
        // from each wave would queue up and stall the waves.
        if constexpr (m < 18 && (m & 1) == 0) copy_piece(std::integral_constant<int, m / 2>{});
        if constexpr (m == 10) start_dp(std::integral_constant<int, 1>{});
        // One wait per two slots: naming the next slot's operand here makes the compiler wait
        // for both now (the statement itself is empty), and the odd slot then needs none.
        if constexpr ((m & 1) == 0) asm volatile("" ::"v"(ring[(m + 1) & 7].v));
        if constexpr (m < 32) {
            constexpr int b = m >> 4, t = (m & 15) >> 1;
            if constexpr (m & 1) score_mfma<kRegV + 4 * t, false>(dp[b], ring[m & 7].v);  // dP - delta = dO V^T - delta
            else score_mfma<kRegK + 4 * t, t == 0>(s[b], ring[m & 7].v);                   // S = Q K^T
        } else {
            constexpr int j = (m - 32) & 15, b = (m - 32) >> 4, half = j >> 3, db = (j & 7) >> 1;
            if constexpr (j & 1) acc_mfma<kAccDK + 16 * db>(ring[m & 7].v, __builtin_bit_cast(bf16x8, dw[b][half]));
            else acc_mfma<kAccDV + 16 * db>(ring[m & 7].v, __builtin_bit_cast(bf16x8, pw[b][half]));
        }
        if constexpr (m >= 16 && m < 48) {
            // slot pair (2j, 2j + 1) of the phase turns accumulator elements 2j, 2j + 1 of
            // block b into packed P and packed dS: the exponentials in the even slot, the
            // rest in the odd one
            constexpr int n = m - 16, b = n >> 4, k = n & 15, j = k >> 1, i = 2 * j;
            // No wait states are needed here: the chain that produced S of block b (k = 0) or dP
            // (k = 1) ended three slots ago, and the two MFMAs issued since then each held the
            // matrix pipeline for as long as an MFMA takes to finish.
            if constexpr ((k & 3) == 0 && n + 4 < 32) Ln = lse4((n + 4) >> 4, ((n + 4) & 15) >> 2);
            if constexpr ((k & 1) == 0) {
                p0 = __builtin_amdgcn_exp2f(fmaf(s[b][i], c, -comp(Lc, i & 3)));
                p1 = __builtin_amdgcn_exp2f(fmaf(s[b][i + 1], c, -comp(Lc, (i + 1) & 3)));
            } else {
                pw[b][j >> 2][j & 3] = FULL ? pack2(p0, p1) : pack2(p0, p1) & mw[b][j];
                const float d0 = p0 * dp[b][i], d1 = p1 * dp[b][i + 1];
                dw[b][j >> 2][j & 3] = FULL ? pack2(d0, d1) : pack2(d0, d1) & mw[b][j];
            }
            if constexpr ((k & 3) == 3) Lc = Ln;
        }
        __builtin_amdgcn_sched_barrier(0);
    });
}

__global__ __launch_bounds__(256) void psattn_dkdv_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sQ[2][kQTileBytes];
    __shared__ __attribute__((aligned(16))) char sG[2][kQTileBytes];  // dO
    __shared__ __attribute__((aligned(16))) float sL[2][64];          // LSE * log2(e)
    __shared__ __attribute__((aligned(16))) float sD[2][64];          // -delta
    // a[0:191] are in use: makes the kernel's register allocation cover them
    asm volatile("" ::: "a0", "a191");
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, c32 = l & 31, g = l >> 5;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const DeviceCsr& csr = a.meta.bwd;
    const RowLaunch rl = csr.launch[blockIdx.x / Hkv];  // one scalar load: row, list bounds, first entry
    const int kvh = blockIdx.x % Hkv, kt = rl.row;
    const int key = kt * 128 + 32 * w + c32;
    const bool kvalid = key < T;
    const int key_hi = kvalid ? a.meta.tok[key].key_hi : 0;  // queries [key, key_hi) read this key
    const size_t koff = (static_cast<size_t>(key) * Hkv + kvh) * 128;

    // K, V fragments of this lane's key -> a[128:191]; dK, dV accumulators a[0:127] = 0
    static_for<0, 8>([&](auto TT) {
        constexpr int t = decltype(TT)::value;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (kvalid) {
            kv = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.K) + koff + 16 * t + 8 * g);
            vv = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.V) + koff + 16 * t + 8 * g);
        }
        acc_set<kRegK + 4 * t + 0>(kv.x);
        acc_set<kRegK + 4 * t + 1>(kv.y);
        acc_set<kRegK + 4 * t + 2>(kv.z);
        acc_set<kRegK + 4 * t + 3>(kv.w);
        acc_set<kRegV + 4 * t + 0>(vv.x);
        acc_set<kRegV + 4 * t + 1>(vv.y);
        acc_set<kRegV + 4 * t + 2>(vv.z);
        acc_set<kRegV + 4 * t + 3>(vv.w);
    });
    static_for<0, 128>([&](auto R) { acc_set<decltype(R)::value>(0u); });

    const float c = a.scale * kLog2e;
    const LaneOffsets lo = lane_offsets(l);
    const int e0 = rl.begin, n_ent = rl.count;
    const int n_it = n_ent * G;

    // Staging of one q-tile (64 rows x 256 B of Q and of dO, 64 LSE * log2 e, 64 delta):
    // asynchronous global -> LDS copies, issued one tile ahead into the buffer the
    // previous tile has just vacated.  Rows past the end of the buffer re-read the
    // last token: whatever they hold is removed by the pair masks (a clipped tile is
    // never FULL).
    const uint32_t row_bytes = static_cast<uint32_t>(Hq) * 256u;
    const DmaLane dml = dma_lane(row_bytes, w, l);
    // The copy of one tile is nine instructions per lane: pieces 0-3 are Q rows, 4-7 dO rows,
    // piece 8 the statistics.  copy_setup fixes the tile, copy_piece issues one piece.
    const char* cp_q = nullptr;   // first Q row of the tile being copied (this head)
    const char* cp_g = nullptr;   // first dO row
    const float* cp_s = nullptr;  // this lane's statistic (waves 0, 1)
    DmaLane cp_lane = dml;
    auto copy_setup = [&](int ent, int h) {
        const int q0 = (ent >> 2) * 64;
        const size_t tile_elems = (static_cast<size_t>(q0) * Hq + h) * 128;
        int rmax = T - 1 - q0;
        cp_q = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.Q) + tile_elems);
        cp_g = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.dO) + tile_elems);
        cp_s = (w ? a.delta : a.lse2) + static_cast<size_t>(h) * T + q0 + min(l, rmax);
        cp_lane = dml;
        if (rmax < 63) {
            asm volatile("; clipped tile" : "+s"(rmax));  // keeps the clamped offsets' arithmetic in this branch
            cp_lane = dma_lane(row_bytes, w, l, rmax);
        }
    };
    auto copy_piece = [&](auto P, auto BUF) {
        constexpr int p = decltype(P)::value, buf = decltype(BUF)::value;
        if constexpr (p < 4) dma16(cp_q, cp_lane.off[p], lds_addr(sQ[buf]) + (16 * w + 4 * p) * kRowBytes);
        else if constexpr (p < 8) dma16(cp_g, cp_lane.off[p - 4], lds_addr(sG[buf]) + (16 * w + 4 * (p - 4)) * kRowBytes);
        else if (w < 2) dma4(cp_s, lds_addr(w ? sD[buf] : sL[buf]));  // wave 0: LSE * log2 e, wave 1: -delta
    };
    // Walk order: q-tiles from the last to the first, and for each q-tile the G heads
    // of the group.  Every k-tile of a sample ends at the same q-tile, so workgroups
    // of neighbouring k-tiles (which run at the same time on the same XCD) read the
    // same Q / dO tile at the same moment and share it through L2.
    EntryStream es;
    es.init(csr.entry, e0 + n_ent - 1, -1, n_ent, l);
    int pk = 0, ph = 0;  // walk position and head (within the group) of the next tile
    int ent = 0, it = 0;
    if (n_it > 0) {
        ent = rl.first_entry;
        copy_setup(ent, kvh * G);
        static_for<0, 9>([&](auto P) { copy_piece(P, std::integral_constant<int, 0>{}); });
        if (++ph == G) { ph = 0; ++pk; }
    }
    // One tile; the buffer index is a compile-time constant, so every LDS address is a lane
    // constant plus an immediate offset.
    auto tile = [&](auto BUF) {
        constexpr int buf = decltype(BUF)::value;
        // this wave's copies of tile `it` have landed; after the barrier every wave's
        // have, and tile it - 1 (same buffer as it + 1) is no longer read
        dma_wait_barrier<0>();
        Frag8 ring[8];
        tile_prefetch(ring, sQ[buf], sG[buf], lo);
        __builtin_amdgcn_sched_barrier(0);
        const int q0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        // After the last tile the copy is issued once more (same tile, other buffer): the slots
        // then need no branch around each piece; nobody reads that buffer.
        if (it + 1 < n_it) {
            if (ph == 0) {  // first head of the next q-tile
                ent = es.get(pk);
                copy_setup(ent, kvh * G);
            } else {        // same q-tile, next head of the group: 128 elements / T statistics further on
                cp_q += 256;
                cp_g += 256;
                cp_s += T;
            }
            if (++ph == G) { ph = 0; ++pk; }
        }
        ++it;
        auto piece = [&](auto P) { copy_piece(P, std::integral_constant<int, buf ^ 1>{}); };
        uint32_t mw[2][8];
        if (full) {
            dkdv_tile<true>(sQ[buf], sG[buf], sL[buf], sD[buf], lo, mw, c, g, ring, piece);
        } else if (__builtin_amdgcn_ballot_w64(max(key, q0) < min(key_hi, q0 + 64)) == 0) {
            // PARTIAL tile none of whose queries reads any of this wave's 32 keys (two of the four
            // waves on the first q-tile of every causal diagonal, and the keys of another sample or
            // response): the wave only issues its share of the next tile's copy
            static_for<0, 9>([&](auto P) { piece(P); });
        } else {
            pair_masks(mw, key - q0, key_hi - q0, g);
            dkdv_tile<false>(sQ[buf], sG[buf], sL[buf], sD[buf], lo, mw, c, g, ring, piece);
        }
    };
    // The K / V loads above have retired before the loop starts, so the loop body holds no
    // wait on a compiler-tracked load (such a wait would also cover the copies in flight).
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    settle();  // the register writes above, before the first MFMA reads them
    while (it < n_it) {
        if (it & 1) tile(std::integral_constant<int, 1>{});
        else tile(std::integral_constant<int, 0>{});
    }
    // no copy may still be writing to LDS when the workgroup ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    settle();  // the last MFMAs, before dK / dV are read out
    if (kvalid) {
        uint16_t* krow = static_cast<uint16_t*>(a.dK) + koff;
        uint16_t* vrow = static_cast<uint16_t*>(a.dV) + koff;
        const float sc = a.scale;
        static_for<0, 16>([&](auto Q4) {
            constexpr int q4 = decltype(Q4)::value, db = q4 >> 2, i4 = q4 & 3;
            const int d = 32 * db + 8 * i4 + 4 * g;
            store4(vrow + d, acc_get<kAccDV + 16 * db + 4 * i4 + 0>(), acc_get<kAccDV + 16 * db + 4 * i4 + 1>(),
                   acc_get<kAccDV + 16 * db + 4 * i4 + 2>(), acc_get<kAccDV + 16 * db + 4 * i4 + 3>());
        });
        if (a.rope) {
            // K arrived rotated: turn dK back by the key's angles (accumulator element 4 i4 + k of block
            // db is head dim 32 db + 8 i4 + 4 g + k; its partner sits in block db + 2)
            const float* trow = a.rope + static_cast<size_t>(rope_position(a.meta.tok[key], key)) * 128;
            static_for<0, 8>([&](auto Q4) {
                constexpr int q4 = decltype(Q4)::value, db = q4 >> 2, i4 = q4 & 3;
                const int d = 32 * db + 8 * i4 + 4 * g;
                const float4 c = *reinterpret_cast<const float4*>(trow + d);
                const float4 s = *reinterpret_cast<const float4*>(trow + 64 + d);
                float l0 = acc_get<kAccDK + 16 * db + 4 * i4 + 0>(), l1 = acc_get<kAccDK + 16 * db + 4 * i4 + 1>(),
                      l2 = acc_get<kAccDK + 16 * db + 4 * i4 + 2>(), l3 = acc_get<kAccDK + 16 * db + 4 * i4 + 3>();
                float h0 = acc_get<kAccDK + 16 * (db + 2) + 4 * i4 + 0>(), h1 = acc_get<kAccDK + 16 * (db + 2) + 4 * i4 + 1>(),
                      h2 = acc_get<kAccDK + 16 * (db + 2) + 4 * i4 + 2>(), h3 = acc_get<kAccDK + 16 * (db + 2) + 4 * i4 + 3>();
                rope_turn<true>(l0, h0, c.x, s.x);
                rope_turn<true>(l1, h1, c.y, s.y);
                rope_turn<true>(l2, h2, c.z, s.z);
                rope_turn<true>(l3, h3, c.w, s.w);
                store4(krow + d, l0 * sc, l1 * sc, l2 * sc, l3 * sc);
                store4(krow + 64 + d, h0 * sc, h1 * sc, h2 * sc, h3 * sc);
            });
        } else {
            static_for<0, 16>([&](auto Q4) {
                constexpr int q4 = decltype(Q4)::value, db = q4 >> 2, i4 = q4 & 3;
                const int d = 32 * db + 8 * i4 + 4 * g;
                store4(krow + d, acc_get<kAccDK + 16 * db + 4 * i4 + 0>() * sc, acc_get<kAccDK + 16 * db + 4 * i4 + 1>() * sc,
                       acc_get<kAccDK + 16 * db + 4 * i4 + 2>() * sc, acc_get<kAccDK + 16 * db + 4 * i4 + 3>() * sc);
            });
        }
    }
}

}  // namespace

int launch_mfma_dkdv(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.bwd.n_rows) * a.Hkv;
    if (grid == 0) return 0;
    psattn_dkdv_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace psattn
