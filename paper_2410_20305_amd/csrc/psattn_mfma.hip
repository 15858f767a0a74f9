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
#include <hip/hip_runtime.h>

#include "psattn_internal.h"

namespace psattn {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kRowBytes = 256;  // 128 bf16

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

struct Stage {  // one thread's share of a 64 x 128 bf16 tile: 4 chunks of 16 bytes
    uint4 c[4];
};

__device__ inline void stage_load(Stage& s, const uint16_t* base, int row0, int T, size_t row_stride,
                                  int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
        const int tok = row0 + row;
        s.c[i] = tok < T ? *reinterpret_cast<const uint4*>(base + static_cast<size_t>(tok) * row_stride + ch * 8)
                         : make_uint4(0, 0, 0, 0);
    }
}

__device__ inline void stage_store(const Stage& s, char* tile, int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
        *reinterpret_cast<uint4*>(tile + tile_off(row, ch)) = s.c[i];
    }
}

__device__ inline void store4(uint16_t* dst, float a, float b, float c, float d) {
    f32x2 v0 = {a, b}, v1 = {c, d};
    union { bf16x2 p[2]; uint2 u; } o;
    o.p[0] = __builtin_convertvector(v0, bf16x2);
    o.p[1] = __builtin_convertvector(v1, bf16x2);
    *reinterpret_cast<uint2*>(dst) = o.u;
}

// ------------------------------------------------------------------ forward
// grid: one workgroup per (q-tile of 128 queries, q-head); 4 waves x 32 queries.
__global__ __launch_bounds__(256, 2) void psattn_fwd_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sK[64 * kRowBytes];
    __shared__ __attribute__((aligned(16))) char sV[64 * kRowBytes];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, g = l >> 5;
    const int T = a.meta.T, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
    const DeviceCsr& csr = a.meta.fwd;
    // heads of one kv group are neighbours in launch order and share an XCD when Hkv == 8
    const int kvh = blockIdx.x % Hkv, rest = blockIdx.x / Hkv;
    const int h = kvh * G + rest % G, qt = csr.order[rest / G];
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

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float c = a.scale * kLog2e;

    int e = csr.row_ptr[qt];
    const int e_end = csr.row_ptr[qt + 1];
    Stage pk, pv;
    int ent = 0;
    if (e < e_end) {
        ent = csr.entry[e];
        stage_load(pk, K, (ent >> 2) * 64, T, kv_stride, tid);
        stage_load(pv, V, (ent >> 2) * 64, T, kv_stride, tid);
    }
    for (; e < e_end; ++e) {
        const int k0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        __syncthreads();
        stage_store(pk, sK, tid);
        stage_store(pv, sV, tid);
        __syncthreads();
        if (e + 1 < e_end) {
            ent = csr.entry[e + 1];
            stage_load(pk, K, (ent >> 2) * 64, T, kv_stride, tid);
            stage_load(pv, V, (ent >> 2) * 64, T, kv_stride, tid);
        }
        // S^T = K Q^T : rows = keys, column = this lane's query
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) s[kb] = mfma(lds_rows(sK, 32 * kb + c32, 2 * t + g), qf[t].v, s[kb]);
        }
        if (!full) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = k0 + 32 * kb + acc_row(i, g);
                    const bool ok = j >= tk.s && j <= q_row && !(j >= tk.hole_lo && j < tk.hole_hi);
                    s[kb][i] = ok ? s[kb][i] : -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m, mx * c);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c, -m_use));
                psum += s[kb][i];
            }
        lsum = lsum * alpha + psum;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        // O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const bf16x8 pb = pack8(s[kb], half);
#pragma unroll
                for (int db = 0; db < 4; ++db)
                    o[db] = mfma(lds_cols(sV, 32 * kb + 16 * half, 32 * db, l), pb, o[db]);
            }
    }
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

// ------------------------------------------------------------------ dQ (q-major)
__global__ __launch_bounds__(256, 2) void psattn_dq_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sK[64 * kRowBytes];
    __shared__ __attribute__((aligned(16))) char sV[64 * kRowBytes];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, g = l >> 5;
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
    const size_t kv_stride = static_cast<size_t>(Hkv) * 128;
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
    const float dl = valid ? a.delta[static_cast<size_t>(h) * T + q_row] : 0.f;
    const float c = a.scale * kLog2e;

    f32x16 dq[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

    int e = csr.row_ptr[qt];
    const int e_end = csr.row_ptr[qt + 1];
    Stage pk, pv;
    int ent = 0;
    if (e < e_end) {
        ent = csr.entry[e];
        stage_load(pk, K, (ent >> 2) * 64, T, kv_stride, tid);
        stage_load(pv, V, (ent >> 2) * 64, T, kv_stride, tid);
    }
    for (; e < e_end; ++e) {
        const int k0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        __syncthreads();
        stage_store(pk, sK, tid);
        stage_store(pv, sV, tid);
        __syncthreads();
        if (e + 1 < e_end) {
            ent = csr.entry[e + 1];
            stage_load(pk, K, (ent >> 2) * 64, T, kv_stride, tid);
            stage_load(pv, V, (ent >> 2) * 64, T, kv_stride, tid);
        }
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
// grid: one workgroup per (k-tile of 128 keys, kv-head); 4 waves x 32 keys.  The
// workgroup walks the G query heads of its group and, for each, the q-tiles
// (64 queries) that can read its keys.
__global__ __launch_bounds__(256) void psattn_dkdv_bf16_mfma(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sQ[64 * kRowBytes];
    __shared__ __attribute__((aligned(16))) char sG[64 * kRowBytes];  // dO
    __shared__ __attribute__((aligned(16))) float sL[64];             // LSE * log2(e)
    __shared__ __attribute__((aligned(16))) float sD[64];             // delta
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, g = l >> 5;
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

    const int e0 = csr.row_ptr[kt], n_ent = csr.row_ptr[kt + 1] - e0;
    const int n_it = n_ent * G;
    Stage pq, pg;
    float pstat = 0.f;  // threads 0..63: LSE of query tid; 64..127: delta of query tid - 64
    int ent = 0, h = kvh * G;
    auto prefetch = [&](int it) {
        ent = csr.entry[e0 + it % n_ent];
        h = kvh * G + it / n_ent;
        const int q0 = (ent >> 2) * 64;
        stage_load(pq, static_cast<const uint16_t*>(a.Q) + h * 128, q0, T, q_stride, tid);
        stage_load(pg, static_cast<const uint16_t*>(a.dO) + h * 128, q0, T, q_stride, tid);
        if (tid < 128) {
            const int qi = q0 + (tid & 63);
            if (tid < 64) pstat = qi < T ? a.LSE[static_cast<size_t>(h) * T + qi] * kLog2e : INFINITY;
            else pstat = qi < T ? a.delta[static_cast<size_t>(h) * T + qi] : 0.f;
        }
    };
    if (n_it > 0) prefetch(0);
    for (int it = 0; it < n_it; ++it) {
        const int q0 = (ent >> 2) * 64;
        const bool full = (ent & 3) == PSATTN_TILE_FULL;
        __syncthreads();
        stage_store(pq, sQ, tid);
        stage_store(pg, sG, tid);
        if (tid < 64) sL[tid] = pstat;
        else if (tid < 128) sD[tid - 64] = pstat;
        __syncthreads();
        if (it + 1 < n_it) prefetch(it + 1);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            f32x16 s, dp;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                s = mfma(lds_rows(sQ, 32 * qb + c32, 2 * t + g), kf[t].v, s);    // S  = Q K^T
                dp = mfma(lds_rows(sG, 32 * qb + c32, 2 * t + g), vf[t].v, dp);  // dP = dO V^T
            }
            f32x16 ds;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int r = 32 * qb + 8 * i4 + 4 * g;
                const float4 ls = *reinterpret_cast<const float4*>(&sL[r]);
                const float4 dl = *reinterpret_cast<const float4*>(&sD[r]);
                const float lsv[4] = {ls.x, ls.y, ls.z, ls.w};
                const float dlv[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = 4 * i4 + j;
                    float p = __builtin_amdgcn_exp2f(fmaf(s[i], c, -lsv[j]));
                    if (!full) {
                        const int q = q0 + r + j;
                        p = (q >= key && q < key_hi) ? p : 0.f;
                    }
                    s[i] = p;
                    ds[i] = p * (dp[i] - dlv[j]);
                }
            }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const bf16x8 pb = pack8(s, half), dsb = pack8(ds, half);
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    dv[db] = mfma(lds_cols(sG, 32 * qb + 16 * half, 32 * db, l), pb, dv[db]);   // dV^T += dO^T P
                    dk[db] = mfma(lds_cols(sQ, 32 * qb + 16 * half, 32 * db, l), dsb, dk[db]);  // dK^T += Q^T dS
                }
            }
        }
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

int launch_mfma_fwd(const AttnArgs& a, void* stream) {
    const unsigned grid = static_cast<unsigned>(a.meta.fwd.n_rows) * a.Hq;
    if (grid == 0) return 0;
    psattn_fwd_bf16_mfma<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a);
    return static_cast<int>(hipGetLastError());
}

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
