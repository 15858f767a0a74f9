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

}  // namespace

int launch_mfma_dq(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    if (grid == 0) return 0;
    psattn_dq_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace psattn
