// bf16 MFMA forward kernels for gfx950; layout and staging helpers are in psattn_mfma_common.h.
#include "psattn_mfma_common.h"

namespace psattn {
namespace {
using namespace mma;

// max(a, b, c); scores are never NaN (the inputs must be finite)
__device__ __forceinline__ float fmax3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// ------------------------------------------------------------------ forward
// grid: one workgroup per (q-tile of 128 queries, q-head); 4 waves x 32 queries.
__global__ __launch_bounds__(256, 2) void psattn_fwd_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sKb[2][64 * kRowBytes];  // double buffered
    __shared__ __attribute__((aligned(16))) char sVb[2][64 * kRowBytes];
    const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, c32 = l & 31, g = l >> 5;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const DeviceCsr& csr = a.meta.fwd;
    // heads of one kv group are neighbours in launch order and share an XCD when Hkv == 8
    const int kvh = blockIdx.x % Hkv, rest = blockIdx.x / Hkv;
    const RowLaunch rl = csr.launch[rest / G];  // one scalar load: row, list bounds, first entry
    const int h = kvh * G + rest % G, qt = rl.row;
    const int q_row = qt * 128 + 32 * w + c32;
    const bool valid = q_row < T;
    Tok4 tk = {kPadStart, 0, 0, 0};
    if (valid) tk = a.meta.tok[q_row];

    const uint16_t* Q = static_cast<const uint16_t*>(a.Q);
    const uint16_t* K = static_cast<const uint16_t*>(a.K) + kvh * 128;
    const uint16_t* V = static_cast<const uint16_t*>(a.V) + kvh * 128;
    const size_t kv_stride = static_cast<size_t>(Hkv) * 128;

    Frag8 qf[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
        qf[t].u = valid ? *reinterpret_cast<const uint4*>(Q + (static_cast<size_t>(q_row) * Hq + h) * 128 + 16 * t + 8 * g)
                        : make_uint4(0, 0, 0, 0);

    if (a.rope) {
        // rotary embedding of this lane's query in registers; the rotated row is also saved for
        // the backward, which streams Q tiles straight into LDS and cannot rotate them on the way
        const float* row = a.rope + static_cast<size_t>(rope_position(tk, q_row)) * 128;
#pragma unroll
        for (int t = 0; t < 4; ++t) rope_frag8(qf[t], qf[t + 4], row, 16 * t + 8 * g);
        if (valid && a.Qr) {
            uint16_t* qr = static_cast<uint16_t*>(a.Qr) + (static_cast<size_t>(q_row) * Hq + h) * 128;
#pragma unroll
            for (int t = 0; t < 8; ++t) *reinterpret_cast<uint4*>(qr + 16 * t + 8 * g) = qf[t].u;
        }
    }
    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float c = a.scale * kLog2e;
    const LaneOffsets lo = lane_offsets(l);
    constexpr int kAhead = 2, kRing = 4;  // measured: 1 and 3 are both slower

    // K / V tiles are copied global -> LDS asynchronously, one tile ahead, into the
    // buffer the previous tile has just vacated; one barrier per tile.
    const uint32_t row_bytes = static_cast<uint32_t>(Hkv) * 256u;
    const char* Kb = reinterpret_cast<const char*>(K);
    const char* Vb = reinterpret_cast<const char*>(V);
    const DmaLane dl = dma_lane(row_bytes, w, l);
    PairCopy pc;
    auto copy_setup = [&](int ent) {
        const int k0 = (ent >> 2) * 64;
        pair_copy_setup(pc, Kb + static_cast<size_t>(k0) * row_bytes, Vb + static_cast<size_t>(k0) * row_bytes, row_bytes,
                        T - 1 - k0, dl, w, l);
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
    // One tile.  The buffer index is a compile-time constant (the loop below is unrolled
    // by two), so every LDS address is a lane constant plus an immediate offset.
    auto tile = [&](auto BUF) {
        constexpr int buf = decltype(BUF)::value;
        // this wave's copies of tile `it` have landed; after the barrier every wave's
        // have, and every wave has left the other buffer
        dma_wait_barrier<0>();
        const int k0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        // The next tile's copy is issued piece by piece, on every other slot of the S phase.  After
        // the last tile the same tile is copied once more (to the other buffer, which nobody
        // reads), so the slots need no branch.
        if (it + 1 < n_ent) {
            ent = es.get(it + 1);
            copy_setup(ent);
        }
        ++it;
        // PARTIAL tile: this lane's allowed elements as a bit mask (the query reads keys
        // [tk.s, q_row] except [hole_lo, hole_hi)).  A wave none of whose 32 queries reads any
        // key of the tile only issues its share of the copy and leaves the SIMD to the other
        // workgroup's wave (two of the four waves on the second tile of every causal diagonal).
        uint32_t bits = 0xffffffffu;
        if (!full) {
            bits = elem_range_bits(tk.s - k0, q_row + 1 - k0, g) & ~elem_range_bits(tk.hole_lo - k0, tk.hole_hi - k0, g);
            if (__builtin_amdgcn_ballot_w64(bits != 0) == 0) {
                static_for<0, 8>([&](auto P) { pair_copy_piece<decltype(P)::value>(pc, sKb[buf ^ 1], sVb[buf ^ 1], w); });
                return;
            }
        }
        const char* sK = sKb[buf];
        const char* sV = sVb[buf];
        // 32 MFMA slots per tile: 0-15 S^T = K Q^T (rows = keys, column = this lane's
        // query), 16-31 O^T += V^T P^T.  The LDS operand of slot m is requested kAhead
        // slots earlier into a register ring.
        Frag8 ring[kRing];
        auto request = [&](auto M) {
            constexpr int m = decltype(M)::value;
            if constexpr (m < 16) {
                constexpr int t = m >> 1, kb = m & 1;
                ring[m % kRing].v = ld_rows<t>(sK + kb * 32 * kRowBytes, lo.nat);
            } else if constexpr (m < 32) {
                constexpr int j = m - 16, kb = j >> 3, half = (j >> 2) & 1, db = j & 3;
                ring[m % kRing].v = ld_cols<db, half>(sV + 32 * kb * kRowBytes, lo.tr1, lo.tr2);
            }
        };
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
        static_for<0, kAhead>([&](auto M) { request(M); });
        static_for<0, 16>([&](auto M) {
            constexpr int m = decltype(M)::value, t = m >> 1, kb = m & 1;
            request(std::integral_constant<int, m + kAhead>{});
            if constexpr ((m & 1) == 0) pair_copy_piece<m / 2>(pc, sKb[buf ^ 1], sVb[buf ^ 1], w);  // every other slot: see PairCopy
            s[kb] = mfma(ring[m % kRing].v, qf[t].v, s[kb]);
            __builtin_amdgcn_sched_barrier(0);
        });
        if (!full) {
            asm volatile("; mask of a PARTIAL tile" ::: "memory");
            static_for<0, 32>([&](auto E) {
                constexpr int e = decltype(E)::value;
                s[e >> 4][e & 15] = keep_or_neg_inf<e>(s[e >> 4][e & 15], bits);
            });
        }
        // The maxima are ordinary compiled code (this file is built with -fno-honor-nans, so that
        // fmaxf(fmaxf(a, b), c) becomes one v_max3_f32 without NaN-quieting instructions): the compiler
        // sees a vector-ALU reader of MFMA results and places the wait states such a reader needs.  (An
        // inline-assembly maximum is not seen as one, and then read scores of the previous tile now and then.)
        // four independent chains each for the maximum and (below) the sum
        float mxp[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) mxp[r] = fmax3(s[0][r], s[1][r], s[0][r + 4]);
#pragma unroll
        for (int r = 0; r < 4; ++r) mxp[r] = fmax3(mxp[r], s[1][r + 4], s[0][r + 8]);
#pragma unroll
        for (int r = 0; r < 4; ++r) mxp[r] = fmax3(mxp[r], s[1][r + 8], s[0][r + 12]);
#pragma unroll
        for (int r = 0; r < 4; ++r) mxp[r] = fmax3(mxp[r], s[1][r + 12], mxp[r]);
        float mx = fmax3(mxp[0], mxp[1], fmax3(mxp[2], mxp[3], mxp[3]));
        mx = fmax3(mx, other_half(mx), mx);
        // Exact running maximum; O and l are rescaled only in tiles where some row's maximum
        // moves (wave ballot).  Letting the reference lag behind the maximum was measured
        // both ways: a fixed lag of 2^8 saves 5 % of this kernel but the largest probability of
        // a row is then no longer exactly 1 and its bf16 rounding shows in O on short rows
        // (0.012 against a bar of 1e-2); a lag bounded by the row's sum so far keeps the
        // accuracy but saves nothing measurable.
        const float m_new = fmaxf(m, mx * c);
        if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
            asm volatile("; rescale" ::: "memory");
            const float m_to = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m - m_to);  // m = -inf: 0 (nothing accumulated yet)
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
            m = m_new;
        }
        const float m_use = m == -INFINITY ? 0.f : m;
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
        bf16x8 pb[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -m_use));
                ps[i & 3] += s[kb][i];
            }
            pb[kb][0] = pack8(s[kb], 0);
            pb[kb][1] = pack8(s[kb], 1);
        }
        const float psum = (ps[0] + ps[1]) + (ps[2] + ps[3]);
        lsum += psum;
        __builtin_amdgcn_sched_barrier(0);
        static_for<16, 32>([&](auto M) {
            constexpr int m_ = decltype(M)::value, j = m_ - 16, kb = j >> 3, half = (j >> 2) & 1, db = j & 3;
            request(std::integral_constant<int, m_ + kAhead>{});
            o[db] = mfma(ring[m_ % kRing].v, pb[kb][half], o[db]);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // Q fragments are in registers before the loop starts, so the loop body holds no wait
    // on a compiler-tracked load (such a wait would also cover the copies in flight)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    while (it + 1 < n_ent) {
        tile(std::integral_constant<int, 0>{});
        tile(std::integral_constant<int, 1>{});
    }
    if (it < n_ent) tile(std::integral_constant<int, 0>{});
    // no copy may still be writing to LDS when the workgroup ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const float l_tot = lsum + other_half(lsum);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (valid) {
        uint16_t* orow = static_cast<uint16_t*>(a.Oout) + (static_cast<size_t>(q_row) * Hq + h) * 128;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4)
                store4(orow + 32 * db + 8 * i4 + 4 * g, o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv,
                       o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv);
        if (g == 0)
            a.LSEout[static_cast<size_t>(h) * T + q_row] = l_tot > 0.f ? m * kLn2 + __logf(l_tot) : -INFINITY;
    }
}

}  // namespace

int launch_mfma_fwd(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    if (grid == 0) return 0;
    psattn_fwd_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

}  // namespace psattn
