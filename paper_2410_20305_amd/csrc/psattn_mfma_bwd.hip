// bf16 MFMA backward (dQ; dK/dV) kernels for gfx950; layout and staging helpers are in psattn_mfma_common.h.
#include "psattn_mfma_common.h"

namespace psattn {
namespace {
using namespace mma;

// ------------------------------------------------------------------ dQ (q-major)
__global__ __launch_bounds__(256, 2) void psattn_dq_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sKb[2][64 * kRowBytes];  // double buffered
    __shared__ __attribute__((aligned(16))) char sVb[2][64 * kRowBytes];
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, c32 = l & 31, g = l >> 5;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const DeviceCsr& csr = a.meta.fwd;
    const int kvh = blockIdx.x % Hkv, rest = blockIdx.x / Hkv;
    const RowLaunch rl = csr.launch[rest / G];  // one scalar load: row, list bounds, first entry
    const int h = kvh * G + rest % G, qt = rl.row;
    const int q_row = qt * 128 + 32 * w + c32;
    const bool valid = q_row < T;
    Tok4 tk = {kPadStart, 0, 0, 0};
    if (valid) tk = a.meta.tok[q_row];

    const uint16_t* K = static_cast<const uint16_t*>(a.K) + kvh * 128;
    const uint16_t* V = static_cast<const uint16_t*>(a.V) + kvh * 128;
    const size_t qoff = (static_cast<size_t>(q_row) * Hq + h) * 128;

    Frag8 qf[8], gf[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        qf[t].u = valid ? *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.Q) + qoff + 16 * t + 8 * g)
                        : make_uint4(0, 0, 0, 0);
        gf[t].u = valid ? *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.dO) + qoff + 16 * t + 8 * g)
                        : make_uint4(0, 0, 0, 0);
    }
    // Rows without keys (padding) have LSE = -inf.  Their scores are masked to -inf below;
    // with +inf here exp2(score - lse2) is 0 for them instead of exp2(-inf + inf).
    const float lse_row = valid ? a.LSE[static_cast<size_t>(h) * T + q_row] : -INFINITY;
    const float lse2 = lse_row == -INFINITY ? INFINITY : lse_row * kLog2e;
    // delta = rowsum(dO o O): this lane holds half of the row's dO already, O is read once
    // here; the result also goes to the workspace for the dK/dV pass that follows
    float dl = 0.f;
    if (valid) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint4 ov = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.O) + qoff + 16 * t + 8 * g);
            const uint32_t ow[4] = {ov.x, ov.y, ov.z, ov.w};
            const uint32_t gw[4] = {gf[t].u.x, gf[t].u.y, gf[t].u.z, gf[t].u.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dl = fmaf(__uint_as_float(ow[j] << 16), __uint_as_float(gw[j] << 16), dl);
                dl = fmaf(__uint_as_float(ow[j] & 0xffff0000u), __uint_as_float(gw[j] & 0xffff0000u), dl);
            }
        }
    }
    dl += other_half(dl);
    if (valid && g == 0) {
        a.delta[static_cast<size_t>(h) * T + q_row] = -dl;  // the dK/dV kernel starts its dP accumulators from -delta
        a.lse2[static_cast<size_t>(h) * T + q_row] = lse2;
    }
    const float c = a.scale * kLog2e;

    f32x16 dq[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

    // K / V tiles are copied global -> LDS asynchronously, one tile ahead, into the
    // buffer the previous tile has just vacated; one barrier per tile.
    const uint32_t row_bytes = static_cast<uint32_t>(Hkv) * 256u;
    const DmaLane dml = dma_lane(row_bytes, w, l);
    PairCopy pc;
    auto copy_setup = [&](int ent) {
        const int k0 = (ent >> 2) * 64;
        pair_copy_setup(pc, reinterpret_cast<const char*>(K) + static_cast<size_t>(k0) * row_bytes,
                        reinterpret_cast<const char*>(V) + static_cast<size_t>(k0) * row_bytes, row_bytes, T - 1 - k0, dml, w, l);
    };
    const int e0 = rl.begin, n_ent = rl.count;
    EntryStream es;
    es.init(csr.entry, e0, 1, n_ent, l);
    int ent = 0, it = 0;
    if (n_ent > 0) {
        ent = rl.first_entry;
        copy_setup(ent);
        static_for<0, 8>([&](auto P) { pair_copy_piece<decltype(P)::value>(pc, sKb[0], sVb[0], w); });
    }
    const LaneOffsets lo = lane_offsets(l);
    constexpr int kAhead = 2, kRing = 4;  // measured: 1 and 3 are both slower
    // One tile = 48 MFMA slots, per block kb of 32 keys:
    //   slots 24 kb +  0-15  S^T = K Q^T and dP^T = V dO^T (alternating)
    //   (dS arithmetic of the block)
    //   slots 24 kb + 16-23  dQ^T += K^T dS^T
    // The LDS operand of slot m is requested kAhead slots earlier into a register ring,
    // across the arithmetic too.  Two workgroups share a CU: the other wave of the SIMD
    // fills the gaps.  The buffer index is a compile-time constant (the loop below is
    // unrolled by two), so every LDS address is a lane constant plus an immediate offset.
    // Only PARTIAL tiles (full == false) run the mask arithmetic.
    auto tile = [&](auto BUF, int k0, bool full) {
        constexpr int buf = decltype(BUF)::value;
        // PARTIAL tile: this lane's allowed elements as a bit mask (the query reads keys
        // [tk.s, q_row] except [hole_lo, hole_hi)).  A wave none of whose 32 queries reads any
        // key of the tile only issues its share of the copy and leaves the SIMD to the other
        // workgroup's wave.
        uint32_t bits = 0xffffffffu;
        // skip32[kb]: none of the wave's 32 queries reads any of the 32 keys of block kb (PARTIAL tiles
        // only): the block's 24 MFMAs and its arithmetic are left out
        bool skip32[2] = {false, false};
        if (!full) {
            bits = elem_range_bits(tk.s - k0, q_row + 1 - k0, g) & ~elem_range_bits(tk.hole_lo - k0, tk.hole_hi - k0, g);
            skip32[0] = __builtin_amdgcn_ballot_w64((bits & 0xffffu) != 0) == 0;
            skip32[1] = __builtin_amdgcn_ballot_w64((bits >> 16) != 0) == 0;
            if (skip32[0]) {  // the next tile's copy rides on the first block's slots: issue it here instead
                static_for<0, 8>([&](auto P) { pair_copy_piece<decltype(P)::value>(pc, sKb[buf ^ 1], sVb[buf ^ 1], w); });
                if (skip32[1]) return;
            }
        }
        const char* sK = sKb[buf];
        const char* sV = sVb[buf];
        Frag8 ring[kRing];
        auto request = [&](auto M) {
            constexpr int m = decltype(M)::value;
            if constexpr (m < 48) {
                constexpr int kb = m / 24, j = m % 24;
                if constexpr (j < 16) {
                    constexpr int t = j >> 1;
                    ring[m % kRing].v = ld_rows<t>(((j & 1) ? sV : sK) + kb * 32 * kRowBytes, lo.nat);
                } else {
                    constexpr int half = (j >> 2) & 1, db = j & 3;
                    ring[m % kRing].v = ld_cols<db, half>(sK + 32 * kb * kRowBytes, lo.tr1, lo.tr2);
                }
            }
        };
        static_for<0, 2>([&](auto KB) {
            constexpr int kb = decltype(KB)::value;
            if (skip32[kb]) return;
            // the first operands of a block are requested by the block before it, unless there is none
            if (kb == 0 || skip32[0]) static_for<0, kAhead>([&](auto M) { request(std::integral_constant<int, 24 * kb + decltype(M)::value>{}); });
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
            static_for<0, 16>([&](auto J) {
                constexpr int j = decltype(J)::value, m = 24 * kb + j, t = j >> 1;
                request(std::integral_constant<int, m + kAhead>{});
                if constexpr (m < 16 && (m & 1) == 0) pair_copy_piece<m / 2>(pc, sKb[buf ^ 1], sVb[buf ^ 1], w);  // every other slot: see PairCopy
                if constexpr (j & 1) dp = mfma(ring[m % kRing].v, gf[t].v, dp);
                else s = mfma(ring[m % kRing].v, qf[t].v, s);
                __builtin_amdgcn_sched_barrier(0);
            });
            if (!full) {
                asm volatile("; mask of a PARTIAL tile" ::: "memory");
                // masked scores become -inf, so p = 0 below
                static_for<0, 16>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    s[i] = keep_or_neg_inf<16 * kb + i>(s[i], bits);
                });
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[i], c, -lse2));
                s[i] = p * (dp[i] - dl);  // dS^T
            }
            bf16x8 dsb[2];
            dsb[0] = pack8(s, 0);
            dsb[1] = pack8(s, 1);
            __builtin_amdgcn_sched_barrier(0);
            static_for<16, 24>([&](auto J) {
                constexpr int j = decltype(J)::value, m = 24 * kb + j, half = (j >> 2) & 1, db = j & 3;
                request(std::integral_constant<int, m + kAhead>{});
                dq[db] = mfma(ring[m % kRing].v, dsb[half], dq[db]);
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };
    auto step = [&](auto BUF) {
        constexpr int buf = decltype(BUF)::value;
        // this wave's copies of tile `it` have landed; after the barrier every wave's
        // have, and every wave has left the other buffer
        dma_wait_barrier<0>();
        const int k0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        // The next tile's copy is issued piece by piece, on every other slot of the first sixteen.
        // After the last tile the same tile is copied once more (to the other buffer, which
        // nobody reads), so the slots need no branch.
        if (it + 1 < n_ent) {
            ent = es.get(it + 1);
            copy_setup(ent);
        }
        ++it;
        tile(BUF, k0, full);
    };
    // every compiler-tracked load and store above has retired before the loop starts, so
    // the loop body holds no wait of the compiler's that would also cover copies in flight
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    while (it + 1 < n_ent) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
    }
    if (it < n_ent) step(std::integral_constant<int, 0>{});
    // no copy may still be writing to LDS when the workgroup ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (a.rope) {
        // Q arrived rotated: what was accumulated is the gradient w.r.t. the rotated query; turning
        // it back by the same angles gives the gradient w.r.t. the unrotated one.  Accumulator
        // element i of block db is head dim 32 db + 8 (i / 4) + 4 g + i % 4; its partner sits in
        // block db + 2 at the same i.
        const float* trow = a.rope + static_cast<size_t>(rope_position(tk, q_row)) * 128;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const float4 c = *reinterpret_cast<const float4*>(trow + 32 * db + 8 * i4 + 4 * g);
                const float4 s = *reinterpret_cast<const float4*>(trow + 64 + 32 * db + 8 * i4 + 4 * g);
                const float cs[4] = {c.x, c.y, c.z, c.w}, sn[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float lo = dq[db][4 * i4 + k], hi = dq[db + 2][4 * i4 + k];
                    rope_turn<true>(lo, hi, cs[k], sn[k]);
                    dq[db][4 * i4 + k] = lo;
                    dq[db + 2][4 * i4 + k] = hi;
                }
            }
    }
    if (valid) {
        uint16_t* row = static_cast<uint16_t*>(a.dQ) + qoff;
        const float sc = a.scale;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4)
                store4(row + 32 * db + 8 * i4 + 4 * g, dq[db][4 * i4] * sc, dq[db][4 * i4 + 1] * sc,
                       dq[db][4 * i4 + 2] * sc, dq[db][4 * i4 + 3] * sc);
    }
}

}  // namespace

int launch_mfma_dq(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    if (grid == 0) return 0;
    psattn_dq_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace psattn
