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
    const int h = kvh * G + rest % G, qt = csr.order[rest / G];
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
    // rows without keys (padding) keep LSE = -inf; every pair of theirs is masked below
    const float lse2 = valid ? a.LSE[static_cast<size_t>(h) * T + q_row] * kLog2e : INFINITY;
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
        a.delta[static_cast<size_t>(h) * T + q_row] = dl;
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
    auto fetch = [&](int ent, int buf) {
        const int k0 = (ent >> 2) * 64;
        dma_tile64(reinterpret_cast<const char*>(K) + static_cast<size_t>(k0) * row_bytes, row_bytes, T - 1 - k0, dml, sKb[buf], w, l);
        dma_tile64(reinterpret_cast<const char*>(V) + static_cast<size_t>(k0) * row_bytes, row_bytes, T - 1 - k0, dml, sVb[buf], w, l);
    };
    const int e0 = csr.row_ptr[qt], n_ent = csr.row_ptr[qt + 1] - e0;
    EntryStream es;
    es.init(csr.entry, e0, 1, n_ent, l);
    int ent = 0, ent_next = 0, buf = 0;
    if (n_ent > 0) {
        ent = es.get(0);
        fetch(ent, 0);
    }
    // every compiler-tracked load and store above has retired before the loop starts, so
    // the loop body holds no wait of the compiler's that would also cover copies in flight
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    for (int it = 0; it < n_ent; ++it, buf ^= 1) {
        // this wave's copies of tile `it` have landed; after the barrier every wave's
        // have, and every wave has left the other buffer
        dma_wait_barrier<0>();
        if (it + 1 < n_ent) {
            ent_next = es.get(it + 1);
            fetch(ent_next, buf ^ 1);
        }
        const int k0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        ent = ent_next;
        const char* sK = sKb[buf];
        const char* sV = sVb[buf];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                s = mfma(lds_rows(sK, 32 * kb + c32, 2 * t + g), qf[t].v, s);    // S^T  = K Q^T
                dp = mfma(lds_rows(sV, 32 * kb + c32, 2 * t + g), gf[t].v, dp);  // dP^T = V dO^T
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float p = __builtin_amdgcn_exp2f(fmaf(s[i], c, -lse2));
                if (!full) {
                    const int j = k0 + 32 * kb + acc_row(i, g);
                    const bool ok = j >= tk.s && j <= q_row && !(j >= tk.hole_lo && j < tk.hole_hi);
                    p = ok ? p : 0.f;
                }
                s[i] = p * (dp[i] - dl);  // dS^T
            }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const bf16x8 dsb = pack8(s, half);
#pragma unroll
                for (int db = 0; db < 4; ++db)
                    dq[db] = mfma(lds_cols(sK, 32 * kb + 16 * half, 32 * db, l), dsb, dq[db]);
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

// ------------------------------------------------------------------ dK, dV (k-major)
// grid: one workgroup per (k-tile of 128 keys, kv-head); 4 waves x 32 keys, one
// wave per SIMD.  The workgroup walks the G query heads of its group and, for
// each, the q-tiles (64 queries) that can read its keys.
//
// With one wave per SIMD nothing hides latency but the wave's own instruction
// stream, so a q-tile is processed as 64 explicitly ordered slots, one MFMA each:
//   slots  0-15  S, dP of queries 0-31
//   slots 16-31  S, dP of queries 32-63      + softmax/dS arithmetic of queries 0-31
//   slots 32-47  dV, dK from queries 0-31    + softmax/dS arithmetic of queries 32-63
//   slots 48-63  dV, dK from queries 32-63
// The LDS operand of slot m is requested kAhead slots earlier into a register
// ring; q-tiles are double buffered in LDS with one barrier per tile.

constexpr int kQTileBytes = 64 * kRowBytes;
constexpr int kAhead = 5;

// Number of accumulator elements e = 16 b + i (b = 32-query block, i = register) of
// lane-half g whose tile row 32 b + acc_row(i, g) lies below x, 0 <= x <= 64.
__device__ inline int elems_below(int x, int g) {
    return 4 * (x >> 3) + min(max((x & 7) - 4 * g, 0), 4);
}

// AND-masks for the packed bf16 pairs (elements 2j, 2j + 1 of block b) of one q-tile:
// the queries allowed to read this lane's key are rows [lo, hi) of the tile.
__device__ inline void pair_masks(uint32_t (&mw)[2][8], bool full, int lo, int hi, int g) {
    uint32_t bits = 0xffffffffu;
    if (!full) {
        const int a = elems_below(min(max(lo, 0), 64), g), b = elems_below(min(max(hi, 0), 64), g);
        bits = static_cast<uint32_t>(((1ull << b) - 1) & ~((1ull << a) - 1));
    }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = 16 * b + 2 * j;
            mw[b][j] = ((bits >> e) & 1u ? 0x0000ffffu : 0u) | ((bits >> (e + 1)) & 1u ? 0xffff0000u : 0u);
        }
}

__device__ inline uint32_t pack2(float a, float b) {
    f32x2 v = {a, b};
    union { bf16x2 p; uint32_t u; } o;
    o.p = __builtin_convertvector(v, bf16x2);
    return o.u;
}

__device__ inline float comp(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

__device__ __forceinline__ void dkdv_tile(const char* sQ, const char* sG, const float* sL, const float* sD,
                                          const LaneOffsets& lo, const Frag8 (&kf)[8], const Frag8 (&vf)[8],
                                          f32x16 (&dk)[4], f32x16 (&dv)[4], const uint32_t (&mw)[2][8],
                                          float c, int g) {
    Frag8 ring[8];
    f32x16 s[2], dp[2];
    u32x4 pw[2][2], dw[2][2];  // packed P and dS of a block: [block][half] is one B operand
    float4 Lc, Dc, Ln, Dn;
    float p0 = 0.f, p1 = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) { s[b][i] = 0.f; dp[b][i] = 0.f; }

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
    auto stats = [&](int b, int i4, float4& L, float4& D) {  // LSE, delta of 4 consecutive queries
        const int r = 32 * b + 8 * i4 + 4 * g;
        L = *reinterpret_cast<const float4*>(sL + r);
        D = *reinterpret_cast<const float4*>(sD + r);
    };

    static_for<0, kAhead>([&](auto M) { request(M); });
    stats(0, 0, Lc, Dc);
    static_for<0, 64>([&](auto M) {
        constexpr int m = decltype(M)::value;
        request(std::integral_constant<int, m + kAhead>{});
        if constexpr (m < 32) {
            constexpr int b = m >> 4, t = (m & 15) >> 1;
            if constexpr (m & 1) dp[b] = mfma(ring[m & 7].v, vf[t].v, dp[b]);
            else s[b] = mfma(ring[m & 7].v, kf[t].v, s[b]);
        } else {
            constexpr int j = (m - 32) & 15, b = (m - 32) >> 4, half = j >> 3, db = (j & 7) >> 1;
            if constexpr (j & 1) dk[db] = mfma(ring[m & 7].v, __builtin_bit_cast(bf16x8, dw[b][half]), dk[db]);
            else dv[db] = mfma(ring[m & 7].v, __builtin_bit_cast(bf16x8, pw[b][half]), dv[db]);
        }
        if constexpr (m >= 16 && m < 48) {
            // slot pair (2j, 2j + 1) of the phase turns accumulator elements 2j, 2j + 1 of
            // block b into packed P (even slot) and packed dS (odd slot)
            constexpr int n = m - 16, b = n >> 4, k = n & 15, j = k >> 1, i = 2 * j;
            if constexpr ((k & 3) == 0 && n + 4 < 32) stats((n + 4) >> 4, ((n + 4) & 15) >> 2, Ln, Dn);
            if constexpr ((k & 1) == 0) {
                p0 = __builtin_amdgcn_exp2f(fmaf(s[b][i], c, -comp(Lc, i & 3)));
                p1 = __builtin_amdgcn_exp2f(fmaf(s[b][i + 1], c, -comp(Lc, (i + 1) & 3)));
                pw[b][j >> 2][j & 3] = pack2(p0, p1) & mw[b][j];
            } else {
                const float d0 = p0 * (dp[b][i] - comp(Dc, i & 3));
                const float d1 = p1 * (dp[b][i + 1] - comp(Dc, (i + 1) & 3));
                dw[b][j >> 2][j & 3] = pack2(d0, d1) & mw[b][j];
            }
            if constexpr ((k & 3) == 3) { Lc = Ln; Dc = Dn; }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
}

__global__ __launch_bounds__(256) void psattn_dkdv_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sQ[2][kQTileBytes];
    __shared__ __attribute__((aligned(16))) char sG[2][kQTileBytes];  // dO
    __shared__ __attribute__((aligned(16))) float sL[2][64];          // LSE * log2(e)
    __shared__ __attribute__((aligned(16))) float sD[2][64];          // delta
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, c32 = l & 31, g = l >> 5;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const DeviceCsr& csr = a.meta.bwd;
    const int kvh = blockIdx.x % Hkv, kt = csr.order[blockIdx.x / Hkv];
    const int key = kt * 128 + 32 * w + c32;
    const bool kvalid = key < T;
    const int key_hi = kvalid ? a.meta.tok[key].key_hi : 0;  // queries [key, key_hi) read this key
    const size_t koff = (static_cast<size_t>(key) * Hkv + kvh) * 128;

    Frag8 kf[8], vf[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        kf[t].u = kvalid ? *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.K) + koff + 16 * t + 8 * g)
                         : make_uint4(0, 0, 0, 0);
        vf[t].u = kvalid ? *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.V) + koff + 16 * t + 8 * g)
                         : make_uint4(0, 0, 0, 0);
    }
    f32x16 dk[4], dv[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk[db][i] = 0.f; dv[db][i] = 0.f; }
    const float c = a.scale * kLog2e;
    const size_t q_stride = static_cast<size_t>(Hq) * 128;
    const LaneOffsets lo = lane_offsets(l);

    const int e0 = csr.row_ptr[kt], n_ent = csr.row_ptr[kt + 1] - e0;
    const int n_it = n_ent * G;

    // Staging of one q-tile (64 rows x 256 B of Q and of dO, 64 LSE * log2 e, 64 delta):
    // asynchronous global -> LDS copies, issued one tile ahead into the buffer the
    // previous tile has just vacated.  Rows past the end of the buffer re-read the
    // last token: whatever they hold is removed by the pair masks (a clipped tile is
    // never FULL).
    const uint32_t row_bytes = static_cast<uint32_t>(Hq) * 256u;
    const DmaLane dml = dma_lane(row_bytes, w, l);
    auto prefetch = [&](int ent, int h, int buf) {
        const int q0 = (ent >> 2) * 64;
        const size_t tile_elems = (static_cast<size_t>(q0) * Hq + h) * 128;
        const int rmax = T - 1 - q0;
        dma_tile64(reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.Q) + tile_elems), row_bytes, rmax, dml, sQ[buf], w, l);
        dma_tile64(reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.dO) + tile_elems), row_bytes, rmax, dml, sG[buf], w, l);
        if (w < 2) {  // wave 0: 64 x LSE * log2 e, wave 1: 64 x delta, one dword per lane
            const float* src = (w ? a.delta : a.lse2) + static_cast<size_t>(h) * T + q0 + min(l, rmax);
            dma4(src, lds_addr(w ? sD[buf] : sL[buf]));
        }
    };
    // Walk order: q-tiles from the last to the first, and for each q-tile the G heads
    // of the group.  Every k-tile of a sample ends at the same q-tile, so workgroups
    // of neighbouring k-tiles (which run at the same time on the same XCD) read the
    // same Q / dO tile at the same moment and share it through L2.
    EntryStream es;
    es.init(csr.entry, e0 + n_ent - 1, -1, n_ent, l);
    int pk = 0, ph = 0;  // walk position and head (within the group) of the next tile
    int ent0 = 0, ent1 = 0;
    if (n_it > 0) {
        ent0 = es.get(0);
        prefetch(ent0, kvh * G, 0);
        if (++ph == G) { ph = 0; ++pk; }
    }
    // K / V fragments are in registers before the loop starts, so the loop body holds no
    // wait on a compiler-tracked load (such a wait would also cover the copies in flight)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    for (int it = 0; it < n_it; ++it) {
        const int buf = it & 1;
        // this wave's copies of tile `it` have landed; after the barrier every wave's
        // have, and tile it - 1 (same buffer as it + 1) is no longer read
        dma_wait_barrier<0>();
        if (it + 1 < n_it) {
            ent1 = es.get(pk);
            prefetch(ent1, kvh * G + ph, buf ^ 1);
            if (++ph == G) { ph = 0; ++pk; }
        }
        const int q0 = (ent0 >> 2) * 64;
        const bool full = (ent0 & 3) == PSATTN_TILE_FULL;
        ent0 = ent1;
        uint32_t mw[2][8];
        pair_masks(mw, full, key - q0, key_hi - q0, g);
        dkdv_tile(sQ[buf], sG[buf], sL[buf], sD[buf], lo, kf, vf, dk, dv, mw, c, g);
    }
    if (kvalid) {
        uint16_t* krow = static_cast<uint16_t*>(a.dK) + koff;
        uint16_t* vrow = static_cast<uint16_t*>(a.dV) + koff;
        const float sc = a.scale;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d = 32 * db + 8 * i4 + 4 * g;
                store4(krow + d, dk[db][4 * i4] * sc, dk[db][4 * i4 + 1] * sc, dk[db][4 * i4 + 2] * sc,
                       dk[db][4 * i4 + 3] * sc);
                store4(vrow + d, dv[db][4 * i4], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]);
            }
    }
}

}  // namespace

int launch_mfma_dq(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    if (grid == 0) return 0;
    psattn_dq_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

int launch_mfma_dkdv(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.bwd.n_rows) * a.Hkv;
    if (grid == 0) return 0;
    psattn_dkdv_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace psattn
