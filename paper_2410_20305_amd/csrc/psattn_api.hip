// C-ABI entry points that touch the device: metadata upload, argument checks and
// kernel dispatch for psattn_fwd / psattn_bwd.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "psattn_internal.h"

using namespace psattn;

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct BlobLayout {
    size_t tok, f_row, f_ent, f_ord, f_lch, b_row, b_ent, b_ord, b_lch, total;
};

BlobLayout layout_of(const psattn_meta& m) {
    BlobLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.tok = take(sizeof(Tok4) * static_cast<size_t>(m.T));
    L.f_row = take(sizeof(int32_t) * m.fwd.row_ptr.size());
    L.f_ent = take(sizeof(int32_t) * m.fwd.idx.size());
    L.f_ord = take(sizeof(int32_t) * m.fwd.order.size());
    L.f_lch = take(sizeof(RowLaunch) * m.fwd.order.size());
    L.b_row = take(sizeof(int32_t) * m.bwd.row_ptr.size());
    L.b_ent = take(sizeof(int32_t) * m.bwd.idx.size());
    L.b_ord = take(sizeof(int32_t) * m.bwd.order.size());
    L.b_lch = take(sizeof(RowLaunch) * m.bwd.order.size());
    L.total = off ? off : 256;
    return L;
}

// walk_backwards: the kernel of this grid starts with the last entry of a row
void fill_csr(char* base, size_t row, size_t ent, size_t ord, size_t lch, const TileCsr& g, bool walk_backwards) {
    std::memcpy(base + row, g.row_ptr.data(), g.row_ptr.size() * sizeof(int32_t));
    int32_t* e = reinterpret_cast<int32_t*>(base + ent);
    for (size_t i = 0; i < g.idx.size(); ++i) e[i] = (g.idx[i] << 2) | g.cls[i];
    std::memcpy(base + ord, g.order.data(), g.order.size() * sizeof(int32_t));
    RowLaunch* rl = reinterpret_cast<RowLaunch*>(base + lch);
    for (size_t i = 0; i < g.order.size(); ++i) {
        const int32_t r = g.order[i], b = g.row_ptr[r], n = g.row_ptr[r + 1] - b;
        rl[i] = RowLaunch{r, b, n, n > 0 ? e[walk_backwards ? b + n - 1 : b] : 0};
    }
}

DeviceCsr view_csr(const char* base, size_t row, size_t ent, size_t ord, size_t lch, const TileCsr& g) {
    DeviceCsr v{};
    v.row_ptr = reinterpret_cast<const int32_t*>(base + row);
    v.entry = reinterpret_cast<const int32_t*>(base + ent);
    v.order = reinterpret_cast<const int32_t*>(base + ord);
    v.launch = reinterpret_cast<const RowLaunch*>(base + lch);
    v.n_rows = static_cast<int32_t>(g.row_ptr.size()) - 1;
    v.tile_q = g.tile_q;
    v.tile_k = g.tile_k;
    return v;
}

// ---- pooled metadata blobs
// A mini-batch needs one pinned staging buffer and one device buffer of the same size.
// Allocating and freeing them every training step would synchronise the device each
// time, so released pairs stay in a small per-process pool and are handed out again.
// A pair carries an event that marks the point after which the device no longer needs
// it (recorded when its meta object is released); it is reused once that event has
// completed.
struct Blob {
    void* d = nullptr;
    void* h = nullptr;
    size_t cap = 0;
    int device = -1;
    hipEvent_t idle = nullptr;  // completes when the previous user is done with d and h
};
constexpr size_t kPoolMax = 8;  // idle pairs kept; beyond that the smallest is freed
std::mutex g_pool_mu;
std::vector<Blob> g_pool;

void destroy_blob(Blob& b) {
    if (b.idle) { (void)hipEventSynchronize(b.idle); (void)hipEventDestroy(b.idle); }
    if (b.d) (void)hipFree(b.d);
    if (b.h) (void)hipHostFree(b.h);
    b = Blob{};
}

// Returns a pair of at least `bytes` on `device`; blocks only if every pooled candidate is
// still in use by the device and the pool is full.
int acquire_blob(size_t bytes, int device, Blob* out) {
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        int best = -1, busy = -1;
        for (size_t i = 0; i < g_pool.size(); ++i) {
            const Blob& b = g_pool[i];
            if (b.device != device || b.cap < bytes) continue;
            if (hipEventQuery(b.idle) == hipSuccess) {
                if (best < 0 || b.cap < g_pool[best].cap) best = static_cast<int>(i);
            } else {
                (void)hipGetLastError();  // hipErrorNotReady is not an error here
                if (busy < 0) busy = static_cast<int>(i);
            }
        }
        if (best < 0 && busy >= 0 && g_pool.size() >= kPoolMax) best = busy;
        if (best >= 0) {
            *out = g_pool[best];
            g_pool.erase(g_pool.begin() + best);
        }
    }
    if (out->d) {
        if (hipEventSynchronize(out->idle) != hipSuccess) { destroy_blob(*out); return PSATTN_EHIP; }
        return PSATTN_OK;
    }
    Blob b;
    b.device = device;
    b.cap = align_up(bytes + bytes / 4, 1 << 16);  // head-room: the next mini-batch differs a little
    if (hipEventCreateWithFlags(&b.idle, hipEventDisableTiming) != hipSuccess) { b.idle = nullptr; (void)hipGetLastError(); return PSATTN_EHIP; }
    if (hipHostMalloc(&b.h, b.cap, hipHostMallocDefault) != hipSuccess) { b.h = nullptr; (void)hipGetLastError(); destroy_blob(b); return PSATTN_ENOMEM; }
    if (hipMalloc(&b.d, b.cap) != hipSuccess) { b.d = nullptr; (void)hipGetLastError(); destroy_blob(b); return PSATTN_ENOMEM; }
    *out = b;
    return PSATTN_OK;
}

// `stream`: the pair may be reused once the work enqueued there so far has finished.
void release_blob(Blob b, hipStream_t stream) {
    if (!b.d) return;
    if (hipEventRecord(b.idle, stream) != hipSuccess) { (void)hipGetLastError(); destroy_blob(b); return; }
    Blob drop;
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        g_pool.push_back(b);
        if (g_pool.size() > kPoolMax) {
            size_t s = 0;
            for (size_t i = 1; i < g_pool.size(); ++i)
                if (g_pool[i].cap < g_pool[s].cap) s = i;
            drop = g_pool[s];
            g_pool.erase(g_pool.begin() + s);
        }
    }
    if (drop.d) destroy_blob(drop);
}

int upload(psattn_meta* m, hipStream_t stream) {
    const BlobLayout L = layout_of(*m);
    if (hipGetDevice(&m->device) != hipSuccess) return PSATTN_EHIP;
    Blob b;
    const int rc = acquire_blob(L.total, m->device, &b);
    if (rc != PSATTN_OK) return rc;
    m->h_stage = b.h;
    m->d_blob = b.d;
    m->blob_cap = b.cap;
    m->blob_idle = b.idle;
    char* h = static_cast<char*>(m->h_stage);
    Tok4* tok = reinterpret_cast<Tok4*>(h + L.tok);
    for (int32_t t = 0; t < m->T; ++t)
        tok[t] = Tok4{m->tok_desc[3 * t], m->tok_desc[3 * t + 1], m->tok_desc[3 * t + 2], m->key_hi[t]};
    fill_csr(h, L.f_row, L.f_ent, L.f_ord, L.f_lch, m->fwd, false);
    fill_csr(h, L.b_row, L.b_ent, L.b_ord, L.b_lch, m->bwd, true);
    if (hipMemcpyAsync(m->d_blob, h, L.total, hipMemcpyHostToDevice, stream) != hipSuccess) {
        (void)hipGetLastError();
        return PSATTN_EHIP;
    }
    const char* d = static_cast<const char*>(m->d_blob);
    m->blob_bytes = L.total;
    m->dev.tok = reinterpret_cast<const Tok4*>(d + L.tok);
    m->dev.fwd = view_csr(d, L.f_row, L.f_ent, L.f_ord, L.f_lch, m->fwd);
    m->dev.bwd = view_csr(d, L.b_row, L.b_ent, L.b_ord, L.b_lch, m->bwd);
    m->dev.T = m->T;
    m->on_device = true;
    return PSATTN_OK;
}

int release_meta(psattn_meta* meta, hipStream_t stream) {
    if (!meta) return PSATTN_OK;
    if (meta->d_blob) {
        Blob b;
        b.d = meta->d_blob; b.h = meta->h_stage; b.cap = meta->blob_cap; b.device = meta->device;
        b.idle = static_cast<hipEvent_t>(meta->blob_idle);
        // the event and the stream belong to the blob's device
        int cur = -1;
        const bool hop = hipGetDevice(&cur) == hipSuccess && cur != b.device;
        if (hop) (void)hipSetDevice(b.device);
        release_blob(b, stream);
        if (hop) (void)hipSetDevice(cur);
    }
    delete meta;
    return PSATTN_OK;
}

int check_common(const psattn_meta* meta, int32_t dt, int32_t Hq, int32_t Hkv, int32_t d) {
    if (!meta) return PSATTN_EINVAL;
    if (dt != PSATTN_F32 && dt != PSATTN_BF16) return PSATTN_EINVAL;
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return PSATTN_EINVAL;
    if (d != 64 && d != 128) return PSATTN_EINVAL;
    if (!meta->on_device) return PSATTN_ENODEVICE;
    // tile * heads products must fit the 1-D grid
    if (static_cast<int64_t>(meta->fwd.n_q_tiles) * Hq > INT32_MAX) return PSATTN_EUNSUPPORTED;
    return PSATTN_OK;
}

// The MFMA kernels fold the scale into a base-2 exponent and take row maxima before
// scaling, which needs scale > 0; anything else runs on the generic kernels.
bool mfma_fwd_ok(const psattn_meta* m, int32_t dt, int32_t d, float scale) {
    return dt == PSATTN_BF16 && d == 128 && scale > 0.f && m->fwd.tile_q == kFwdTileQ &&
           m->fwd.tile_k == kFwdTileK;
}
bool mfma_bwd_ok(const psattn_meta* m, int32_t dt, int32_t d, float scale) {
    return mfma_fwd_ok(m, dt, d, scale) && m->bwd.tile_q == kBwdTileQ && m->bwd.tile_k == kBwdTileK;
}

// ---- optional per-pass event timing
bool g_profile = false;
struct EventPair { hipEvent_t a, b; int pass; };
std::vector<EventPair> g_events;
constexpr size_t kMaxPendingEvents = 1 << 16;

struct PassTimer {
    hipStream_t stream;
    EventPair ev{};
    bool active = false;
    PassTimer(int pass, void* s) : stream(static_cast<hipStream_t>(s)) {
        if (!g_profile) return;
        if (hipEventCreate(&ev.a) != hipSuccess) return;
        if (hipEventCreate(&ev.b) != hipSuccess) { (void)hipEventDestroy(ev.a); return; }
        ev.pass = pass;
        active = hipEventRecord(ev.a, stream) == hipSuccess;
    }
    ~PassTimer() {
        if (!active) return;
        (void)hipEventRecord(ev.b, stream);
        if (g_events.size() < kMaxPendingEvents) {
            g_events.push_back(ev);
        } else {  // nobody reads them: do not grow without bound
            (void)hipEventDestroy(ev.a);
            (void)hipEventDestroy(ev.b);
        }
    }
};

// kernel launched last per pass (psattn_kernel_name)
const char* g_last_kernel[4] = {nullptr, nullptr, nullptr, nullptr};

}  // namespace

namespace psattn {

size_t bwd_scratch_bytes(const psattn_meta* meta, int32_t n_q_heads) {
    return 2 * align_up(sizeof(float) * static_cast<size_t>(meta->T) * n_q_heads, 256) + 256;
}

int bwd_checked(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                float scale, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                const float* LSE, void* dQ, void* dK, void* dV, void* scratch_base, size_t scratch_bytes,
                void* hip_stream, const float* rope_table) {
    const int rc = check_common(meta, dt, n_q_heads, n_kv_heads, head_dim);
    if (rc != PSATTN_OK) return rc;
    if (meta->T == 0) return PSATTN_OK;
    if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV || !scratch_base) return PSATTN_EINVAL;
    if (scratch_bytes < bwd_scratch_bytes(meta, n_q_heads)) return PSATTN_EINVAL;
    AttnArgs a{};
    a.meta = meta->dev;
    a.Hq = n_q_heads; a.Hkv = n_kv_heads; a.d = head_dim; a.scale = scale;
    a.Q = Q; a.K = K; a.V = V; a.O = O; a.dO = dO; a.LSE = LSE;
    a.dQ = dQ; a.dK = dK; a.dV = dV;
    a.rope = rope_table;
    a.delta = reinterpret_cast<float*>(align_up(reinterpret_cast<uintptr_t>(scratch_base), 256));
    a.lse2 = a.delta + align_up(sizeof(float) * static_cast<size_t>(meta->T) * n_q_heads, 256) / sizeof(float);
    int err = 0;
    const bool mfma = mfma_bwd_ok(meta, dt, head_dim, scale);
    if (rope_table && !mfma) return PSATTN_EUNSUPPORTED;  // rotary embedding lives in the matrix-core kernels only
    if (!mfma) {  // the MFMA dQ kernel computes delta itself and leaves it in the scratch
        PassTimer t(1, hip_stream);
        err = launch_delta(dt, a, hip_stream);
        g_last_kernel[1] = "delta_kernel";
    }
    if (err) return PSATTN_EHIP;
    {
        PassTimer t(2, hip_stream);
        err = mfma ? launch_mfma_dq(a, hip_stream) : launch_generic_dq(dt, a, hip_stream);
        g_last_kernel[2] = mfma ? "psattn_dq_bf16_mfma" : "generic_dq";
    }
    if (err) return PSATTN_EHIP;
    {
        PassTimer t(3, hip_stream);
        err = mfma ? launch_mfma_dkdv(a, hip_stream) : launch_generic_dkdv(dt, a, hip_stream);
        g_last_kernel[3] = mfma ? "psattn_dkdv_bf16_mfma" : "generic_dkdv";
    }
    return err == 0 ? PSATTN_OK : PSATTN_EHIP;
}

int fwd_checked(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                float scale, const void* Q, const void* K, const void* V, void* O, float* LSE,
                const float* rope_table, void* Qr, void* hip_stream) {
    int rc = check_common(meta, dt, n_q_heads, n_kv_heads, head_dim);
    if (rc != PSATTN_OK) return rc;
    if (meta->T == 0) return PSATTN_OK;
    if (!Q || !K || !V || !O || !LSE) return PSATTN_EINVAL;
    AttnArgs a{};
    a.meta = meta->dev;
    a.Hq = n_q_heads; a.Hkv = n_kv_heads; a.d = head_dim; a.scale = scale;
    a.Q = Q; a.K = K; a.V = V; a.Oout = O; a.LSEout = LSE;
    a.rope = rope_table; a.Qr = Qr;
    const bool mfma = mfma_fwd_ok(meta, dt, head_dim, scale);
    if (rope_table && !mfma) return PSATTN_EUNSUPPORTED;  // rotary embedding lives in the matrix-core kernels only
    int err;
    {
        PassTimer t(0, hip_stream);
        err = mfma ? launch_mfma_fwd(a, hip_stream) : launch_generic_fwd(dt, a, hip_stream);
        g_last_kernel[0] = mfma ? "psattn_fwd_bf16_mfma" : "generic_fwd";
    }
    return err == 0 ? PSATTN_OK : PSATTN_EHIP;
}

}  // namespace psattn

extern "C" {

int psattn_profile_enable(int32_t on) {
    g_profile = on != 0;
    return PSATTN_OK;
}

int psattn_profile_read(double* sum_ms, int64_t* count) {
    if (!sum_ms || !count) return PSATTN_EINVAL;
    for (int i = 0; i < 4; ++i) { sum_ms[i] = 0.0; count[i] = 0; }
    int rc = PSATTN_OK;
    for (EventPair& e : g_events) {
        float ms = 0.f;
        if (hipEventSynchronize(e.b) != hipSuccess || hipEventElapsedTime(&ms, e.a, e.b) != hipSuccess) rc = PSATTN_EHIP;
        else { sum_ms[e.pass] += ms; count[e.pass]++; }
        (void)hipEventDestroy(e.a);
        (void)hipEventDestroy(e.b);
    }
    g_events.clear();
    return rc;
}

int psattn_build_meta(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                      const int32_t* chosen_len, const int32_t* rejected_len, int32_t total_tokens,
                      int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                      void* hip_stream, psattn_meta** out) {
    psattn_meta* m = nullptr;
    int rc = build_host(n_samples, offset, prefix_len, chosen_len, rejected_len, total_tokens, tile_q,
                        tile_k, bwd_tile_q, bwd_tile_k, &m);
    if (rc != PSATTN_OK) return rc;
    rc = upload(m, static_cast<hipStream_t>(hip_stream));
    if (rc != PSATTN_OK) {
        release_meta(m, static_cast<hipStream_t>(hip_stream));
        *out = nullptr;
        return rc;
    }
    *out = m;
    return PSATTN_OK;
}

int psattn_build_meta_multi(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                            const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                            int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                            void* hip_stream, psattn_meta** out) {
    psattn_meta* m = nullptr;
    int rc = build_host_multi(n_samples, offset, prefix_len, resp_ptr, resp_len, total_tokens, tile_q, tile_k,
                              bwd_tile_q, bwd_tile_k, &m);
    if (rc != PSATTN_OK) return rc;
    rc = upload(m, static_cast<hipStream_t>(hip_stream));
    if (rc != PSATTN_OK) {
        release_meta(m, static_cast<hipStream_t>(hip_stream));
        *out = nullptr;
        return rc;
    }
    *out = m;
    return PSATTN_OK;
}

int psattn_free_meta(psattn_meta* meta) { return release_meta(meta, nullptr); }

int psattn_free_meta_async(psattn_meta* meta, void* hip_stream) {
    return release_meta(meta, static_cast<hipStream_t>(hip_stream));
}

int psattn_trim_pool(void) {
    std::vector<Blob> all;
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        all.swap(g_pool);
    }
    int cur = -1;
    (void)hipGetDevice(&cur);
    for (Blob& b : all) {
        if (cur >= 0 && b.device != cur) (void)hipSetDevice(b.device);
        destroy_blob(b);
        if (cur >= 0 && b.device != cur) (void)hipSetDevice(cur);
    }
    return PSATTN_OK;
}

int psattn_uses_mfma(const psattn_meta* meta, int32_t dt, int32_t head_dim, float scale, int32_t backward) {
    if (!meta) return PSATTN_EINVAL;
    return (backward ? mfma_bwd_ok(meta, dt, head_dim, scale) : mfma_fwd_ok(meta, dt, head_dim, scale)) ? 1 : 0;
}

int psattn_fwd(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
               int32_t head_dim, float scale, const void* Q, const void* K, const void* V, void* O,
               float* LSE, void* hip_stream) {
    return fwd_checked(meta, dt, n_q_heads, n_kv_heads, head_dim, scale, Q, K, V, O, LSE, nullptr, nullptr, hip_stream);
}

size_t psattn_bwd_workspace_bytes(const psattn_meta* meta, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim) {
    (void)n_kv_heads; (void)head_dim;
    if (!meta || n_q_heads <= 0) return 0;
    return bwd_scratch_bytes(meta, n_q_heads);
}

int psattn_bwd(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
               int32_t head_dim, float scale, const void* Q, const void* K, const void* V,
               const void* O, const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
               void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bwd_checked(meta, dt, n_q_heads, n_kv_heads, head_dim, scale, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace,
                       workspace_bytes, hip_stream);
}

const char* psattn_kernel_name(int32_t dt, int32_t pass) {
    if (pass < 0 || pass > 3) return "";
    if (g_last_kernel[pass]) return g_last_kernel[pass];
    const bool bf = dt == PSATTN_BF16;
    switch (pass) {
        case 0: return bf ? "psattn_fwd_bf16_mfma" : "generic_fwd";
        case 1: return "delta_kernel";
        case 2: return bf ? "psattn_dq_bf16_mfma" : "generic_dq";
        default: return bf ? "psattn_dkdv_bf16_mfma" : "generic_dkdv";
    }
}

}  // extern "C"
