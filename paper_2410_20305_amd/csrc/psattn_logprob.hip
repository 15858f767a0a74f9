// Per-response log-probabilities and the DPO loss over prefix-shared sequences
// (paper Section 2.1, Eq. 1: the loss needs log pi(y | x) of every completion).
//
// In the prefix-shared sequence [prompt | response 1 | ... | response k] the logits row of a
// token predicts the next token of that token's own branch: inside a response the following
// token, and the LAST prompt token predicts the first token of every response.  Prompt rows
// other than the last, the last row of every response and padding predict nothing and are
// never read, which is where the prefix sharing saves work here too (the prompt is most of
// the tokens).
//
// All three passes stream logits rows of `vocab` elements and are bound by HBM bandwidth:
// one workgroup per row, 16-byte loads, online max / sum in fp32, one exponential per element.
// Every sum is taken in a fixed order (no atomics): results are deterministic.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "psattn.h"

struct psattn_lp_plan {
    int32_t T = 0, n_samples = 0, n_resp = 0, n_rows = 0;
    int64_t n_items = 0;
    int device = -1;
    void* d_blob = nullptr;
    // device views into d_blob
    const int32_t* rows = nullptr;         // [n_rows]   logits rows that predict something, ascending
    const int32_t* row_desc = nullptr;     // [T]        -1: predicts nothing; j >= 0: row inside response j (predicts token row + 1);
                                           //            -2 - i: last prompt row of sample i (predicts the first token of each response)
    const int32_t* resp_first = nullptr;   // [n_resp]   first token of the response
    const int32_t* resp_len = nullptr;     // [n_resp]
    const int32_t* resp_prev = nullptr;    // [n_resp]   last prompt row of its sample, -1 if the prompt is empty
    const int32_t* samp_ptr = nullptr;     // [n_samples + 1] responses of sample i
};

namespace {

constexpr int kThreads = 256;

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ inline uint16_t f32_to_bf16(float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
__device__ inline float ld1(const float* p) { return *p; }
__device__ inline float ld1(const uint16_t* p) { return bf16_to_f32(*p); }
__device__ inline void st1(float* p, float v) { *p = v; }
__device__ inline void st1(uint16_t* p, float v) { *p = f32_to_bf16(v); }

template <typename E> struct Vec;
template <> struct Vec<uint16_t> { static constexpr int N = 8; };  // 16 bytes
template <> struct Vec<float> { static constexpr int N = 4; };

__device__ inline void load_vec(const uint16_t* p, float (&x)[8]) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[2 * j] = __uint_as_float(w[j] << 16);
        x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
}
__device__ inline void load_vec(const float* p, float (&x)[4]) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
}
__device__ inline void store_vec(uint16_t* p, const float (&x)[8]) {
    uint4 u;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = static_cast<uint32_t>(f32_to_bf16(x[2 * j])) | (static_cast<uint32_t>(f32_to_bf16(x[2 * j + 1])) << 16);
    u.x = w[0]; u.y = w[1]; u.z = w[2]; u.w = w[3];
    *reinterpret_cast<uint4*>(p) = u;
}
__device__ inline void store_vec(float* p, const float (&x)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
}

// (m, s) pairs of an online log-sum-exp: value = m + log s
__device__ inline void lse_merge(float& m, float& s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    if (mn == -INFINITY) { m = mn; s = 0.f; return; }
    s = s * __expf(m - mn) + s2 * __expf(m2 - mn);
    m = mn;
}

// block-wide reduction in a fixed order; result valid in thread 0
__device__ inline void block_lse(float& m, float& s, float* sm, float* ss) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_down(m, off), s2 = __shfl_down(s, off);
        lse_merge(m, s, m2, s2);
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sm[w] = m; ss[w] = s; }
    __syncthreads();
    if (threadIdx.x == 0)
        for (int i = 1; i < kThreads / 64; ++i) lse_merge(m, s, sm[i], ss[i]);
}

__device__ inline float block_sum(float v, float* sm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) sm[w] = v;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int i = 1; i < kThreads / 64; ++i) v += sm[i];
    return v;
}

// ---- pass 1: log-sum-exp of every row that predicts something
template <typename E>
__global__ __launch_bounds__(kThreads) void psattn_lp_row_lse(const int32_t* rows, int vocab, const E* logits, float* row_lse) {
    __shared__ float sm[kThreads / 64], ss[kThreads / 64];
    const int row = rows[blockIdx.x];
    const E* x = logits + static_cast<size_t>(row) * vocab;
    constexpr int N = Vec<E>::N;
    float m = -INFINITY, s = 0.f;
    const int n_vec = (vocab % N == 0) ? vocab / N : 0;  // rows are 16-byte aligned only then
    for (int c = threadIdx.x; c < n_vec; c += kThreads) {
        float v[N];
        load_vec(x + static_cast<size_t>(c) * N, v);
        float mx = v[0];
#pragma unroll
        for (int j = 1; j < N; ++j) mx = fmaxf(mx, v[j]);
        const float mn = fmaxf(m, mx);
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < N; ++j) acc += __expf(v[j] - mn);
        s = s * __expf(m - mn) + acc;
        m = mn;
    }
    for (int c = n_vec * N + threadIdx.x; c < vocab; c += kThreads) {
        const float v = ld1(x + c), mn = fmaxf(m, v);
        s = s * __expf(m - mn) + __expf(v - mn);
        m = mn;
    }
    block_lse(m, s, sm, ss);
    if (threadIdx.x == 0) row_lse[row] = m + __logf(s);
}

// ---- pass 2: log pi(response | prompt) = sum over its tokens of logit[row, token] - lse[row]
template <typename E>
__global__ __launch_bounds__(kThreads) void psattn_lp_resp_sum(const int32_t* resp_first, const int32_t* resp_len,
                                                               const int32_t* resp_prev, int vocab, const E* logits,
                                                               const int32_t* token_ids, const float* row_lse, float* resp_logp) {
    __shared__ float sm[kThreads / 64];
    const int j = blockIdx.x, first = resp_first[j], n = resp_len[j], prev = resp_prev[j];
    float acc = 0.f;
    for (int u = threadIdx.x; u < n; u += kThreads) {
        const int row = u == 0 ? prev : first + u - 1;
        if (row < 0) continue;  // empty prompt: nothing predicts the first token
        const int tok = token_ids[first + u];
        if (tok < 0 || tok >= vocab) continue;  // not a token of this vocabulary: contributes nothing
        acc += ld1(logits + static_cast<size_t>(row) * vocab + tok) - row_lse[row];
    }
    acc = block_sum(acc, sm);
    if (threadIdx.x == 0) resp_logp[j] = acc;
}

// ---- backward: d logits = sum over the row's items of d_logp[j] (onehot(target) - softmax(row))
template <typename E>
__global__ __launch_bounds__(kThreads) void psattn_lp_bwd(const int32_t* row_desc, const int32_t* resp_first,
                                                          const int32_t* resp_len, const int32_t* samp_ptr, int vocab,
                                                          const E* logits, const int32_t* token_ids, const float* row_lse,
                                                          const float* d_logp, E* dlogits) {
    const int row = blockIdx.x, desc = row_desc[row];
    const E* x = logits + static_cast<size_t>(row) * vocab;
    E* g = dlogits + static_cast<size_t>(row) * vocab;
    constexpr int N = Vec<E>::N;
    const int n_vec = (vocab % N == 0) ? vocab / N : 0;
    if (desc == -1) {  // predicts nothing: the row of the gradient is zero, the logits are not read
        float z[N];
#pragma unroll
        for (int j = 0; j < N; ++j) z[j] = 0.f;
        for (int c = threadIdx.x; c < n_vec; c += kThreads) store_vec(g + static_cast<size_t>(c) * N, z);
        for (int c = n_vec * N + threadIdx.x; c < vocab; c += kThreads) st1(g + c, 0.f);
        return;
    }
    // total weight of the row's items
    int r0, r1;
    if (desc >= 0) { r0 = desc; r1 = desc + 1; }
    else { const int i = -2 - desc; r0 = samp_ptr[i]; r1 = samp_ptr[i + 1]; }
    // target token of item j of this row, -1 if the item does not exist (empty response) or its token
    // is not of this vocabulary
    auto target = [&](int j) {
        if (desc < 0 && resp_len[j] == 0) return -1;
        const int t = desc >= 0 ? token_ids[row + 1] : token_ids[resp_first[j]];
        return t >= 0 && t < vocab ? t : -1;
    };
    float coef = 0.f;
    for (int j = r0; j < r1; ++j)
        if (target(j) >= 0) coef += d_logp[j];
    const float lse = row_lse[row];
    for (int c = threadIdx.x; c < n_vec; c += kThreads) {
        float v[N];
        load_vec(x + static_cast<size_t>(c) * N, v);
#pragma unroll
        for (int j = 0; j < N; ++j) v[j] = -coef * __expf(v[j] - lse);
        store_vec(g + static_cast<size_t>(c) * N, v);
    }
    for (int c = n_vec * N + threadIdx.x; c < vocab; c += kThreads) st1(g + c, -coef * __expf(ld1(x + c) - lse));
    // the target columns: recomputed whole by one thread after the block's stores are visible, so
    // each is rounded once and two responses that start with the same token add up
    __threadfence_block();
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int j = r0; j < r1; ++j) {
            const int tgt = target(j);
            if (tgt < 0) continue;
            float v = -coef * __expf(ld1(x + tgt) - lse);
            for (int k = r0; k < r1; ++k)
                if (target(k) == tgt) v += d_logp[k];
            st1(g + tgt, v);
        }
    }
}

// ---- DPO loss of (chosen, rejected) pairs and its derivative w.r.t. the policy log-probabilities
__global__ void psattn_dpo_loss_kernel(int n_pairs, float beta, const float* lp, const float* lr, float* loss, float* d_lp) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const float z = beta * ((lp[2 * i] - lr[2 * i]) - (lp[2 * i + 1] - lr[2 * i + 1]));
    // -log sigmoid(z) = max(-z, 0) + log1p(exp(-|z|))
    loss[i] = fmaxf(-z, 0.f) + log1pf(expf(-fabsf(z)));
    const float dz = -1.f / (1.f + expf(z));
    if (d_lp) { d_lp[2 * i] = beta * dz; d_lp[2 * i + 1] = -beta * dz; }
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

extern "C" {

int psattn_logprob_plan(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len, const int32_t* resp_ptr,
                        const int32_t* resp_len, int32_t total_tokens, void* hip_stream, psattn_lp_plan** out) {
    if (!out) return PSATTN_EINVAL;
    *out = nullptr;
    if (n_samples < 0 || total_tokens < 0) return PSATTN_EINVAL;
    if (n_samples > 0 && (!offset || !prefix_len || !resp_ptr)) return PSATTN_EINVAL;
    try {
        const int32_t n_resp = n_samples > 0 ? resp_ptr[n_samples] : 0;
        if (n_samples > 0 && (resp_ptr[0] != 0 || n_resp < 0 || (n_resp > 0 && !resp_len))) return PSATTN_EINVAL;
        std::vector<int32_t> row_desc(static_cast<size_t>(total_tokens), -1), rows, first(n_resp), len(n_resp), prev(n_resp);
        int64_t prev_end = 0, n_items = 0;
        for (int32_t i = 0; i < n_samples; ++i) {
            const int64_t o = offset[i], p = prefix_len[i];
            if (o < 0 || p < 0 || resp_ptr[i + 1] < resp_ptr[i]) return PSATTN_EINVAL;
            if (o < prev_end) return PSATTN_EOVERLAP;
            int64_t t = o + p;
            bool any = false;
            for (int32_t j = resp_ptr[i]; j < resp_ptr[i + 1]; ++j) {
                const int64_t n = resp_len[j];
                if (n < 0) return PSATTN_EINVAL;
                if (t + n > total_tokens) return PSATTN_ERANGE;
                first[j] = static_cast<int32_t>(t);
                len[j] = static_cast<int32_t>(n);
                prev[j] = p > 0 ? static_cast<int32_t>(o + p - 1) : -1;
                for (int64_t u = 0; u + 1 < n; ++u) row_desc[t + u] = j;  // predicts token t + u + 1
                n_items += n - (p > 0 || n == 0 ? 0 : 1);
                any = any || n > 0;
                t += n;
            }
            if (t == o) return PSATTN_EINVAL;
            if (t > total_tokens) return PSATTN_ERANGE;
            if (p > 0 && any) row_desc[o + p - 1] = -2 - i;
            prev_end = t;
        }
        for (int32_t t = 0; t < total_tokens; ++t)
            if (row_desc[t] != -1) rows.push_back(t);
        psattn_lp_plan* pl = new psattn_lp_plan();
        pl->T = total_tokens; pl->n_samples = n_samples; pl->n_resp = n_resp;
        pl->n_rows = static_cast<int32_t>(rows.size()); pl->n_items = n_items;
        // one blob: rows | row_desc | first | len | prev | samp_ptr
        size_t off = 0;
        auto take = [&](size_t n) { const size_t o = off; off = align_up(off + n * sizeof(int32_t), 256); return o; };
        const size_t o_rows = take(rows.size()), o_desc = take(row_desc.size()), o_first = take(n_resp), o_len = take(n_resp),
                     o_prev = take(n_resp), o_ptr = take(static_cast<size_t>(n_samples) + 1);
        std::vector<char> host(off ? off : 256, 0);
        auto put = [&](size_t o, const int32_t* src, size_t n) { if (n) std::memcpy(host.data() + o, src, n * sizeof(int32_t)); };
        put(o_rows, rows.data(), rows.size());
        put(o_desc, row_desc.data(), row_desc.size());
        put(o_first, first.data(), n_resp);
        put(o_len, len.data(), n_resp);
        put(o_prev, prev.data(), n_resp);
        if (n_samples > 0) put(o_ptr, resp_ptr, static_cast<size_t>(n_samples) + 1);
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        if (hipGetDevice(&pl->device) != hipSuccess || hipMalloc(&pl->d_blob, host.size()) != hipSuccess) {
            (void)hipGetLastError();
            delete pl;
            return PSATTN_ENOMEM;
        }
        // the host vector dies with this call, so the copy has to be complete on return
        if (hipMemcpyAsync(pl->d_blob, host.data(), host.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(pl->d_blob);
            delete pl;
            return PSATTN_EHIP;
        }
        const char* d = static_cast<const char*>(pl->d_blob);
        pl->rows = reinterpret_cast<const int32_t*>(d + o_rows);
        pl->row_desc = reinterpret_cast<const int32_t*>(d + o_desc);
        pl->resp_first = reinterpret_cast<const int32_t*>(d + o_first);
        pl->resp_len = reinterpret_cast<const int32_t*>(d + o_len);
        pl->resp_prev = reinterpret_cast<const int32_t*>(d + o_prev);
        pl->samp_ptr = reinterpret_cast<const int32_t*>(d + o_ptr);
        *out = pl;
    } catch (const std::bad_alloc&) {
        return PSATTN_ENOMEM;
    }
    return PSATTN_OK;
}

int psattn_logprob_plan_free(psattn_lp_plan* plan) {
    if (!plan) return PSATTN_OK;
    int rc = PSATTN_OK;
    if (plan->d_blob && hipFree(plan->d_blob) != hipSuccess) rc = PSATTN_EHIP;
    delete plan;
    return rc;
}

int psattn_logprob_plan_info(const psattn_lp_plan* plan, int32_t* n_responses, int32_t* n_rows, int64_t* n_items) {
    if (!plan) return PSATTN_EINVAL;
    if (n_responses) *n_responses = plan->n_resp;
    if (n_rows) *n_rows = plan->n_rows;
    if (n_items) *n_items = plan->n_items;
    return PSATTN_OK;
}

int psattn_logprob_fwd(const psattn_lp_plan* plan, int32_t dt, int32_t vocab, const void* logits, const int32_t* token_ids,
                       float* row_lse, float* resp_logp, void* hip_stream) {
    if (!plan || vocab <= 0 || (dt != PSATTN_F32 && dt != PSATTN_BF16)) return PSATTN_EINVAL;
    if (plan->n_resp == 0) return PSATTN_OK;
    if (!logits || !token_ids || !row_lse || !resp_logp) return PSATTN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (plan->n_rows > 0) {
        if (dt == PSATTN_BF16) psattn_lp_row_lse<uint16_t><<<plan->n_rows, kThreads, 0, s>>>(plan->rows, vocab, static_cast<const uint16_t*>(logits), row_lse);
        else psattn_lp_row_lse<float><<<plan->n_rows, kThreads, 0, s>>>(plan->rows, vocab, static_cast<const float*>(logits), row_lse);
    }
    if (dt == PSATTN_BF16) psattn_lp_resp_sum<uint16_t><<<plan->n_resp, kThreads, 0, s>>>(plan->resp_first, plan->resp_len, plan->resp_prev, vocab, static_cast<const uint16_t*>(logits), token_ids, row_lse, resp_logp);
    else psattn_lp_resp_sum<float><<<plan->n_resp, kThreads, 0, s>>>(plan->resp_first, plan->resp_len, plan->resp_prev, vocab, static_cast<const float*>(logits), token_ids, row_lse, resp_logp);
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}

int psattn_logprob_bwd(const psattn_lp_plan* plan, int32_t dt, int32_t vocab, const void* logits, const int32_t* token_ids,
                       const float* row_lse, const float* d_resp_logp, void* dlogits, void* hip_stream) {
    if (!plan || vocab <= 0 || (dt != PSATTN_F32 && dt != PSATTN_BF16)) return PSATTN_EINVAL;
    if (plan->T == 0) return PSATTN_OK;
    if (!logits || !token_ids || !row_lse || !dlogits || (plan->n_resp > 0 && !d_resp_logp)) return PSATTN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (dt == PSATTN_BF16) psattn_lp_bwd<uint16_t><<<plan->T, kThreads, 0, s>>>(plan->row_desc, plan->resp_first, plan->resp_len, plan->samp_ptr, vocab, static_cast<const uint16_t*>(logits), token_ids, row_lse, d_resp_logp, static_cast<uint16_t*>(dlogits));
    else psattn_lp_bwd<float><<<plan->T, kThreads, 0, s>>>(plan->row_desc, plan->resp_first, plan->resp_len, plan->samp_ptr, vocab, static_cast<const float*>(logits), token_ids, row_lse, d_resp_logp, static_cast<float*>(dlogits));
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}

int psattn_dpo_loss(int32_t n_pairs, float beta, const float* logp_policy, const float* logp_ref, float* loss, float* d_logp,
                    void* hip_stream) {
    if (n_pairs < 0) return PSATTN_EINVAL;
    if (n_pairs == 0) return PSATTN_OK;
    if (!logp_policy || !logp_ref || !loss) return PSATTN_EINVAL;
    psattn_dpo_loss_kernel<<<(n_pairs + 255) / 256, 256, 0, static_cast<hipStream_t>(hip_stream)>>>(n_pairs, beta, logp_policy, logp_ref, loss, d_logp);
    return hipGetLastError() == hipSuccess ? PSATTN_OK : PSATTN_EHIP;
}

}  // extern "C"
