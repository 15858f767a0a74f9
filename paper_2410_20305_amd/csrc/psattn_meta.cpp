// Host metadata builder: per-token descriptors and the two block masks.
//
// The block mask is what Section 3.1 of the paper computes once per mini-batch
// and hands to every attention layer: blocks without any allowed pair are
// skipped.  Here it is derived by interval arithmetic from the sample table
// (prompt / chosen / rejected lengths); the T x T boolean mask of Algorithms 1
// and 3 is never materialised.  Integer only.
#include <algorithm>
#include <cstring>
#include <memory>
#include <new>

#include "psattn_internal.h"

namespace psattn {
namespace {

constexpr int32_t kSmallGridRows = 256;

inline int64_t tri(int64_t n) { return n * (n + 1) / 2; }

// #{(q, k): qa <= q < qb, ka <= k < kb, k <= q}
int64_t causal_pairs(int64_t qa, int64_t qb, int64_t ka, int64_t kb) {
    if (qa >= qb || ka >= kb) return 0;
    // rows q < ka see nothing; rows q >= kb - 1 see all kb - ka keys; between: q + 1 - ka
    int64_t lo = std::max(qa, ka), hi = std::min(qb, kb - 1);
    int64_t n = 0;
    if (lo < hi) n += tri(hi - ka) - tri(lo - ka);  // sum_{q=lo}^{hi-1} (q + 1 - ka)
    int64_t full_from = std::max(qa, kb - 1);
    if (full_from < qb) n += (qb - full_from) * (kb - ka);
    return n;
}

// A sample is [prompt | response 1 | ... | response k]; resp[j] is the first token of
// response j + 1, resp[k] == e.  The paper's case is k = 2 (chosen, rejected).
struct Sample {
    int64_t o, C, e;          // start, first token behind the prompt, end
    const int64_t* resp;      // k + 1 ascending positions, resp[0] == C
    int32_t k;
};

inline int64_t overlap(int64_t a0, int64_t a1, int64_t b0, int64_t b1) {
    return std::max<int64_t>(0, std::min(a1, b1) - std::max(a0, b0));
}

// Allowed pairs of one sample inside the rectangle [qa, qb) x [ka, kb).  Everything not
// later than the query is allowed (Algorithm 1's causal clause) except, for a query in
// response j, the keys of the responses before it: they form one range [C, start of
// response j) and all lie before the query, so each removes one causal pair.
int64_t sample_pairs(const Sample& s, int64_t qa, int64_t qb, int64_t ka, int64_t kb) {
    qa = std::max(qa, s.o);
    qb = std::min(qb, s.e);
    ka = std::max(ka, s.o);
    kb = std::min(kb, s.e);
    if (qa >= qb || ka >= kb) return 0;
    int64_t n = causal_pairs(qa, qb, ka, kb);
    if (s.k >= 2 && qb > s.resp[1] && kb > s.C) {
        // responses that hold a query of the range, from the second response on
        int32_t j = static_cast<int32_t>(std::upper_bound(s.resp, s.resp + s.k + 1, qa) - s.resp) - 1;
        for (j = std::max(j, 1); j < s.k && s.resp[j] < qb; ++j)
            n -= overlap(qa, qb, s.resp[j], s.resp[j + 1]) * overlap(ka, kb, s.C, s.resp[j]);
    }
    return n;
}

// false: more non-skipped tiles than the int32 row pointers can count
bool classify(const std::vector<Sample>& samples, int64_t T, int32_t tq, int32_t tk, TileCsr& g) {
    g.tile_q = tq;
    g.tile_k = tk;
    g.n_q_tiles = static_cast<int32_t>((T + tq - 1) / tq);
    g.n_k_tiles = static_cast<int32_t>((T + tk - 1) / tk);
    g.row_ptr.assign(g.n_q_tiles + 1, 0);
    g.idx.clear();
    g.cls.clear();
    std::vector<int64_t> cnt;
    size_t first = 0;  // first sample that may still intersect the current q-tile
    for (int32_t a = 0; a < g.n_q_tiles; ++a) {
        const int64_t q0 = static_cast<int64_t>(a) * tq, q1 = std::min<int64_t>(T, q0 + tq);
        while (first < samples.size() && samples[first].e <= q0) ++first;
        size_t last = first;
        while (last < samples.size() && samples[last].o < q1) ++last;
        if (first < last) {
            const int64_t kt_lo = samples[first].o / tk;
            const int64_t kt_hi = (q1 - 1) / tk;  // keys never lie after the last query
            cnt.assign(kt_hi - kt_lo + 1, 0);
            for (size_t i = first; i < last; ++i) {
                const Sample& s = samples[i];
                const int64_t qb = std::min(q1, s.e);
                for (int64_t b = s.o / tk; b <= (qb - 1) / tk; ++b)
                    cnt[b - kt_lo] += sample_pairs(s, q0, q1, b * tk, std::min<int64_t>(T, (b + 1) * tk));
            }
            for (int64_t b = kt_lo; b <= kt_hi; ++b) {
                const int64_t n = cnt[b - kt_lo];
                if (n == 0) continue;
                const bool unclipped = (q0 + tq <= T) && ((b + 1) * tk <= T);
                const bool full = unclipped && n == static_cast<int64_t>(tq) * tk;
                g.idx.push_back(static_cast<int32_t>(b));
                g.cls.push_back(full ? PSATTN_TILE_FULL : PSATTN_TILE_PARTIAL);
            }
        }
        if (g.idx.size() > static_cast<size_t>(INT32_MAX)) return false;
        g.row_ptr[a + 1] = static_cast<int32_t>(g.idx.size());
    }
    return true;
}

// rows <-> columns of a CSR (counting sort keeps indices ascending inside a row)
void transpose(const TileCsr& in, TileCsr& out) {
    out.tile_q = in.tile_q;
    out.tile_k = in.tile_k;
    out.n_q_tiles = in.n_q_tiles;
    out.n_k_tiles = in.n_k_tiles;
    const int32_t n_rows = in.n_k_tiles;
    out.row_ptr.assign(n_rows + 1, 0);
    for (int32_t b : in.idx) out.row_ptr[b + 1]++;
    for (int32_t b = 0; b < n_rows; ++b) out.row_ptr[b + 1] += out.row_ptr[b];
    out.idx.resize(in.idx.size());
    out.cls.resize(in.cls.size());
    std::vector<int32_t> fill(out.row_ptr.begin(), out.row_ptr.end() - 1);
    for (int32_t a = 0; a < in.n_q_tiles; ++a)
        for (int32_t e = in.row_ptr[a]; e < in.row_ptr[a + 1]; ++e) {
            const int32_t pos = fill[in.idx[e]]++;
            out.idx[pos] = a;
            out.cls[pos] = in.cls[e];
        }
}

// Launch order of the rows.
//
// Large grids: rows of one sample that are neighbours in this order run at the same
// time and stream the same tiles of the other operand, so they should stay
// neighbours (the L2 of an XCD then serves most of their reads), and inside a sample
// the long rows should come first.  Causality gives both: a q-tile late in its sample
// has the longest k-list, a k-tile early in its sample the longest q-list.  So q-major
// rows run from the last tile to the first, k-major rows from the first to the last.
//
// Small grids (fewer rows than a couple of waves of workgroups): there is little to
// share and the tail dominates, so rows are simply sorted longest first.
void order_rows(TileCsr& g, bool descending) {
    const int32_t n = static_cast<int32_t>(g.row_ptr.size()) - 1;
    g.order.resize(n);
    for (int32_t i = 0; i < n; ++i) g.order[i] = descending ? n - 1 - i : i;
    if (n < kSmallGridRows)
        std::stable_sort(g.order.begin(), g.order.end(), [&](int32_t x, int32_t y) {
            return g.row_ptr[x + 1] - g.row_ptr[x] > g.row_ptr[y + 1] - g.row_ptr[y];
        });
}

}  // namespace

int build_host_multi(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                     const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                     int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                     psattn_meta** out) {
    if (!out) return PSATTN_EINVAL;
    *out = nullptr;
    if (n_samples < 0 || total_tokens < 0) return PSATTN_EINVAL;
    if (n_samples > 0 && (!offset || !prefix_len || !resp_ptr)) return PSATTN_EINVAL;
    if (tile_q < 0 || tile_k < 0 || bwd_tile_q < 0 || bwd_tile_k < 0) return PSATTN_EINVAL;
    if (tile_q == 0) tile_q = kFwdTileQ;
    if (tile_k == 0) tile_k = kFwdTileK;
    if (bwd_tile_q == 0) bwd_tile_q = kBwdTileQ;
    if (bwd_tile_k == 0) bwd_tile_k = kBwdTileK;
    const int64_t T = total_tokens;
    // a list entry packs (tile index << 2 | class) into an int32
    constexpr int64_t kMaxTiles = int64_t{1} << 29;
    for (int32_t t : {tile_q, tile_k, bwd_tile_q, bwd_tile_k})
        if ((T + t - 1) / t >= kMaxTiles) return PSATTN_EUNSUPPORTED;
    std::vector<Sample> samples;
    std::vector<int64_t> starts;  // response boundaries of all samples, k + 1 per sample
    int64_t prev_end = 0, n_allowed = 0, n_positions = 0;
    try {
        samples.reserve(n_samples);
        if (n_samples > 0) {
            if (resp_ptr[0] != 0) return PSATTN_EINVAL;
            for (int32_t i = 0; i < n_samples; ++i)
                if (resp_ptr[i + 1] < resp_ptr[i]) return PSATTN_EINVAL;
            if (resp_ptr[n_samples] > 0 && !resp_len) return PSATTN_EINVAL;
            starts.reserve(static_cast<size_t>(resp_ptr[n_samples]) + n_samples);
        }
        std::vector<size_t> first(n_samples);
        for (int32_t i = 0; i < n_samples; ++i) {
            const int64_t o = offset[i], p = prefix_len[i];
            if (o < 0 || p < 0) return PSATTN_EINVAL;
            if (o < prev_end) return PSATTN_EOVERLAP;
            first[i] = starts.size();
            int64_t t = o + p;
            n_allowed += tri(p);
            starts.push_back(t);
            for (int32_t j = resp_ptr[i]; j < resp_ptr[i + 1]; ++j) {
                const int64_t r = resp_len[j];
                if (r < 0) return PSATTN_EINVAL;
                t += r;
                if (t > T) return PSATTN_ERANGE;
                n_allowed += r * p + tri(r);
                n_positions = std::max(n_positions, p + r);  // every response counts on from the prompt's length
                starts.push_back(t);
            }
            n_positions = std::max(n_positions, p);
            if (t == o) return PSATTN_EINVAL;  // empty sample
            if (t > T) return PSATTN_ERANGE;
            samples.push_back({o, o + p, t, nullptr, resp_ptr[i + 1] - resp_ptr[i]});
            prev_end = t;
        }
        for (int32_t i = 0; i < n_samples; ++i) samples[i].resp = starts.data() + first[i];
        std::unique_ptr<psattn_meta> m(new psattn_meta());
        m->T = total_tokens;
        m->n_samples = n_samples;
        m->n_allowed = n_allowed;
        m->n_positions = static_cast<int32_t>(n_positions);
        m->tok_desc.assign(static_cast<size_t>(3) * T, 0);
        m->key_hi.assign(T, 0);
        for (int64_t t = 0; t < T; ++t) m->tok_desc[3 * t] = kPadStart;
        for (const Sample& s : samples) {
            for (int64_t t = s.o; t < s.C; ++t) {
                m->tok_desc[3 * t] = static_cast<int32_t>(s.o);
                m->key_hi[t] = static_cast<int32_t>(s.e);  // a prompt key is visible to the whole sample
            }
            for (int32_t j = 0; j < s.k; ++j)
                for (int64_t t = s.resp[j]; t < s.resp[j + 1]; ++t) {
                    m->tok_desc[3 * t] = static_cast<int32_t>(s.o);
                    if (j >= 1) {  // must not see the responses before its own: keys [C, start of response j)
                        m->tok_desc[3 * t + 1] = static_cast<int32_t>(s.C);
                        m->tok_desc[3 * t + 2] = static_cast<int32_t>(s.resp[j]);
                    }
                    // a response key is visible up to the end of its own response only
                    m->key_hi[t] = static_cast<int32_t>(s.resp[j + 1]);
                }
        }
        if (!classify(samples, T, tile_q, tile_k, m->fwd)) return PSATTN_EUNSUPPORTED;
        order_rows(m->fwd, true);
        TileCsr qmajor;
        if (!classify(samples, T, bwd_tile_q, bwd_tile_k, qmajor)) return PSATTN_EUNSUPPORTED;
        transpose(qmajor, m->bwd);
        order_rows(m->bwd, false);
        *out = m.release();
    } catch (const std::bad_alloc&) {
        return PSATTN_ENOMEM;
    }
    return PSATTN_OK;
}

// The paper's format: two responses per prompt, chosen then rejected.
int build_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
               const int32_t* chosen_len, const int32_t* rejected_len, int32_t total_tokens,
               int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
               psattn_meta** out) {
    if (!out) return PSATTN_EINVAL;
    *out = nullptr;
    if (n_samples < 0) return PSATTN_EINVAL;
    if (n_samples > 0 && (!chosen_len || !rejected_len)) return PSATTN_EINVAL;
    try {
        std::vector<int32_t> ptr(static_cast<size_t>(n_samples) + 1), len(static_cast<size_t>(n_samples) * 2);
        for (int32_t i = 0; i < n_samples; ++i) {
            ptr[i] = 2 * i;
            len[2 * i] = chosen_len[i];
            len[2 * i + 1] = rejected_len[i];
        }
        ptr[n_samples] = 2 * n_samples;
        return build_host_multi(n_samples, offset, prefix_len, ptr.data(), len.data(), total_tokens, tile_q, tile_k,
                                bwd_tile_q, bwd_tile_k, out);
    } catch (const std::bad_alloc&) {
        return PSATTN_ENOMEM;
    }
}

}  // namespace psattn

extern "C" {

int psattn_build_meta_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                           const int32_t* chosen_len, const int32_t* rejected_len,
                           int32_t total_tokens, int32_t tile_q, int32_t tile_k,
                           int32_t bwd_tile_q, int32_t bwd_tile_k, psattn_meta** out) {
    return psattn::build_host(n_samples, offset, prefix_len, chosen_len, rejected_len, total_tokens,
                              tile_q, tile_k, bwd_tile_q, bwd_tile_k, out);
}

int psattn_build_meta_multi_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                                 const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                                 int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                                 psattn_meta** out) {
    return psattn::build_host_multi(n_samples, offset, prefix_len, resp_ptr, resp_len, total_tokens, tile_q, tile_k,
                                    bwd_tile_q, bwd_tile_k, out);
}

int psattn_meta_tiles(const psattn_meta* meta, int32_t grid, int32_t* tile_q, int32_t* tile_k,
                      int32_t* n_q_tiles, int32_t* n_k_tiles, int64_t* n_entries) {
    if (!meta || (grid != PSATTN_GRID_FWD && grid != PSATTN_GRID_BWD)) return PSATTN_EINVAL;
    const psattn::TileCsr& g = grid == PSATTN_GRID_FWD ? meta->fwd : meta->bwd;
    if (tile_q) *tile_q = g.tile_q;
    if (tile_k) *tile_k = g.tile_k;
    if (n_q_tiles) *n_q_tiles = g.n_q_tiles;
    if (n_k_tiles) *n_k_tiles = g.n_k_tiles;
    if (n_entries) *n_entries = static_cast<int64_t>(g.idx.size());
    return PSATTN_OK;
}

int psattn_meta_copy_csr(const psattn_meta* meta, int32_t grid, int32_t* row_ptr, int32_t* idx,
                         uint8_t* cls) {
    if (!meta || (grid != PSATTN_GRID_FWD && grid != PSATTN_GRID_BWD)) return PSATTN_EINVAL;
    const psattn::TileCsr& g = grid == PSATTN_GRID_FWD ? meta->fwd : meta->bwd;
    if (!row_ptr || ((!idx || !cls) && !g.idx.empty())) return PSATTN_EINVAL;
    std::memcpy(row_ptr, g.row_ptr.data(), g.row_ptr.size() * sizeof(int32_t));
    if (!g.idx.empty()) {
        std::memcpy(idx, g.idx.data(), g.idx.size() * sizeof(int32_t));
        std::memcpy(cls, g.cls.data(), g.cls.size());
    }
    return PSATTN_OK;
}

int psattn_meta_copy_tok_desc(const psattn_meta* meta, int32_t* tok_desc) {
    if (!meta || (!tok_desc && meta->T > 0)) return PSATTN_EINVAL;
    if (meta->T > 0) std::memcpy(tok_desc, meta->tok_desc.data(), meta->tok_desc.size() * sizeof(int32_t));
    return PSATTN_OK;
}

int psattn_meta_copy_key_desc(const psattn_meta* meta, int32_t* key_hi) {
    if (!meta || (!key_hi && meta->T > 0)) return PSATTN_EINVAL;
    if (meta->T > 0) std::memcpy(key_hi, meta->key_hi.data(), meta->key_hi.size() * sizeof(int32_t));
    return PSATTN_OK;
}

int psattn_meta_copy_positions(const psattn_meta* meta, int32_t* pos, int32_t* n_positions) {
    if (!meta || (!pos && meta->T > 0)) return PSATTN_EINVAL;
    for (int32_t t = 0; t < meta->T; ++t) {
        const int32_t s = meta->tok_desc[3 * t];
        // the hidden key range lies between the prompt and the token's own response: skipping it
        // puts the response right behind the prompt
        pos[t] = s == psattn::kPadStart ? 0 : t - s - (meta->tok_desc[3 * t + 2] - meta->tok_desc[3 * t + 1]);
    }
    if (n_positions) *n_positions = meta->n_positions;
    return PSATTN_OK;
}

int psattn_meta_allowed_pairs(const psattn_meta* meta, int64_t* n_allowed) {
    if (!meta || !n_allowed) return PSATTN_EINVAL;
    *n_allowed = meta->n_allowed;
    return PSATTN_OK;
}

const char* psattn_strerror(int status) {
    switch (status) {
        case PSATTN_OK: return "ok";
        case PSATTN_EINVAL: return "invalid argument";
        case PSATTN_EOVERLAP: return "samples unsorted or overlapping";
        case PSATTN_ERANGE: return "sample reaches beyond total_tokens";
        case PSATTN_ENOMEM: return "out of memory";
        case PSATTN_EHIP: return "HIP runtime error";
        case PSATTN_EUNSUPPORTED: return "unsupported configuration";
        case PSATTN_ENODEVICE: return "metadata has no device copy";
        case PSATTN_ELIMIT: return "request exceeds a fixed capacity of this entry point";
        default: return "unknown status";
    }
}

}  // extern "C"
