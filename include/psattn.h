/*
 * psattn — prefix-shared DPO attention for MI355X (gfx950), C ABI.
 *
 * One packed token buffer holds samples laid out as [prompt | chosen | rejected]
 * (paper Section 3.1); several samples may share the buffer, with padding between
 * or after them (Section 3.2, Section 4.3.2).  Attention is ordinary causal
 * softmax attention restricted by the prefix-sharing mask of Algorithm 1, in its
 * packed form of Algorithm 3:
 *
 *     allowed(q, kv) = kv <= q  &&  doc(q) == doc(kv)
 *                      && !(R <= q && C <= kv < R)
 *
 * where C / R are the first chosen / rejected token of q's sample.  A sample with
 * chosen_len = rejected_len = 0 is a plain causal document, which expresses the
 * paper's baseline formats (Algorithm 2, the "normal paired format").
 *
 * The paper's (b, q) batch/position coordinates map to the flat token index
 * b * L + q; rows are independent under the document clause, so a flat buffer with
 * sample offsets covers both unpacked batches and packed, padded rows.
 *
 * Conventions
 *   - every function returns PSATTN_OK (0) or a negative psattn_status; nothing
 *     aborts or throws; psattn_strerror() names a code.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the current device.  The caller owns every tensor and the stream;
 *     the library owns only the psattn_meta objects (host arrays + a pinned staging
 *     buffer and a device buffer taken from a small pool inside the library).
 *   - hip_stream is a hipStream_t passed as void* (NULL = the null stream).  All
 *     device work is enqueued on it and is asynchronous.  Calls that may block the
 *     host or synchronise the device: psattn_build_meta only when it has to allocate a
 *     new buffer pair (the first mini-batches of a process, or a mini-batch larger than
 *     any before) or when all pooled pairs are still in use by the device;
 *     psattn_trim_pool; psattn_profile_read.  psattn_fwd, psattn_bwd,
 *     psattn_free_meta and psattn_free_meta_async never block and never allocate.
 *   - tensors are contiguous, token-major: Q, O, dO, dQ are [T, n_q_heads, head_dim],
 *     K, V, dK, dV are [T, n_kv_heads, head_dim], head_dim fastest.  LSE is
 *     [n_q_heads, T] float.  q-heads [g*G, (g+1)*G), G = n_q_heads / n_kv_heads,
 *     read kv-head g.
 *   - padding tokens (covered by no sample) are never attended to; every output at
 *     a padding position is written as zero (LSE = -inf).  Outputs are overwritten,
 *     never accumulated into.  The input VALUES at padding positions must be finite:
 *     the matrix-core kernels multiply them by exact zeros, and 0 * inf or 0 * NaN
 *     would reach real tokens of the same tile.
 */
#ifndef PSATTN_H
#define PSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct psattn_meta psattn_meta; /* opaque */
typedef struct psattn_rope psattn_rope; /* opaque: rotary-embedding table on one device */
typedef struct psattn_lp_plan psattn_lp_plan; /* opaque: which logits rows predict which tokens */

typedef enum {
    PSATTN_OK = 0,
    PSATTN_EINVAL = -1,       /* null pointer, negative length, empty sample, bad heads / head_dim / tiles */
    PSATTN_EOVERLAP = -2,     /* samples not sorted by offset, or overlapping */
    PSATTN_ERANGE = -3,       /* a sample reaches beyond total_tokens */
    PSATTN_ENOMEM = -4,       /* host or device allocation failed */
    PSATTN_EHIP = -5,         /* a HIP runtime call failed */
    PSATTN_EUNSUPPORTED = -6, /* valid request this build has no kernel for */
    PSATTN_ENODEVICE = -7,    /* meta was built host-only; no device copy to run kernels from */
    PSATTN_ELIMIT = -8        /* request exceeds a fixed capacity of the entry point called */
} psattn_status;

typedef enum { PSATTN_F32 = 0, PSATTN_BF16 = 1 } psattn_dtype;

/* tile classes of the block mask */
enum { PSATTN_TILE_SKIPPED = 0, PSATTN_TILE_PARTIAL = 1, PSATTN_TILE_FULL = 2 };

/* which tile grid of a meta object */
enum { PSATTN_GRID_FWD = 0, /* q-major CSR, used by psattn_fwd and the dQ pass  */
       PSATTN_GRID_BWD = 1  /* k-major CSR, used by the dK/dV pass              */ };

/*
 * Build the block mask for one mini-batch (Section 3.1: computed once per training
 * step and reused by every attention layer and head).
 *
 * Samples: sample i covers flat tokens [offset[i], offset[i] + prefix_len[i] +
 * chosen_len[i] + rejected_len[i]).  Samples must be sorted by offset and must not
 * overlap; gaps and a tail are padding.  Each of the three lengths may be zero but
 * not all three.  n_samples may be zero (everything is padding).
 *
 * Two tile grids over the flat buffer are classified, tile t = tokens
 * [t*tile, min((t+1)*tile, T)):
 *   FWD grid (tile_q x tile_k), stored q-major: for each q-tile the ascending list
 *       of k-tiles that are not SKIPPED, with their class;
 *   BWD grid (bwd_tile_q x bwd_tile_k), stored k-major: for each k-tile the
 *       ascending list of q-tiles that are not SKIPPED.
 * SKIPPED = no allowed pair; FULL = the unclipped rectangle lies inside the buffer
 * and every pair is allowed (a kernel needs neither mask nor bounds check);
 * PARTIAL = the rest.  A tile size of 0 selects the library default (the size the
 * bf16 kernels are built for).  The cost is O(T + non-skipped tiles); the T x T mask
 * is never materialised.
 *
 * Also derived: per-token descriptors (s, hole_lo, hole_hi): s = first token of the
 * token's sample (INT32_MAX for padding); [hole_lo, hole_hi) = [C, R) for tokens of
 * the rejected response, (0, 0) otherwise.  allowed(q, kv) == (s_q <= kv <= q &&
 * !(hole_lo_q <= kv < hole_hi_q)).
 *
 * psattn_build_meta uploads the metadata to the current device with one
 * asynchronous copy on hip_stream (the host staging buffer stays alive inside the
 * object).  Tile grids with 2^29 or more tiles along an axis, or more than
 * INT32_MAX non-skipped tiles, are refused with PSATTN_EUNSUPPORTED.  psattn_build_meta_host builds the same object without touching any
 * device (for inspection and planning); kernels refuse it with PSATTN_ENODEVICE.
 * On error *out is set to NULL.
 */
int psattn_build_meta(int32_t n_samples,
                      const int32_t* offset,       /* host [n_samples] */
                      const int32_t* prefix_len,   /* host [n_samples] */
                      const int32_t* chosen_len,   /* host [n_samples] */
                      const int32_t* rejected_len, /* host [n_samples] */
                      int32_t total_tokens,        /* T, including padding */
                      int32_t tile_q, int32_t tile_k,
                      int32_t bwd_tile_q, int32_t bwd_tile_k,
                      void* hip_stream,
                      psattn_meta** out);

int psattn_build_meta_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                           const int32_t* chosen_len, const int32_t* rejected_len,
                           int32_t total_tokens, int32_t tile_q, int32_t tile_k,
                           int32_t bwd_tile_q, int32_t bwd_tile_k, psattn_meta** out);

/*
 * The same block mask for samples with any number of responses per prompt,
 * [prompt | response 1 | ... | response k]: every response attends to the prompt and
 * to itself, never to another response (Section 2.2 relates the prefix-sharing mask to
 * tree-structured attention masks: the prompt is the trunk, the responses are
 * branches).  k = 2 is the paper's [prompt | chosen | rejected]; k = 1 and k = 0 are
 * plain causal documents.  The responses of sample i have lengths
 * resp_len[resp_ptr[i] .. resp_ptr[i + 1]) (host arrays, resp_ptr[0] = 0, CSR style).
 * Per-token descriptors: tokens of response j >= 2 get (hole_lo, hole_hi) = (first token
 * behind the prompt, first token of response j), everything else (0, 0).  Everything
 * else (grids, errors, upload, ownership) is as for psattn_build_meta, and the object is
 * used with the same psattn_fwd / psattn_bwd.
 */
int psattn_build_meta_multi(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                            const int32_t* resp_ptr, /* host [n_samples + 1] */
                            const int32_t* resp_len, /* host [resp_ptr[n_samples]] */
                            int32_t total_tokens, int32_t tile_q, int32_t tile_k,
                            int32_t bwd_tile_q, int32_t bwd_tile_k, void* hip_stream, psattn_meta** out);
int psattn_build_meta_multi_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                                 const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                                 int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                                 psattn_meta** out);

/* Releases the object; its buffers return to the library's pool.  The caller must
 * make sure no kernel that uses it is still running.  NULL is accepted. */
int psattn_free_meta(psattn_meta* meta);

/* Stream-ordered release for training loops: the object is gone when the call returns,
 * its buffers are handed out again only after all work enqueued on hip_stream before
 * this call has finished.  Never blocks.  (Section 3.1: one block mask per training
 * step; a loop builds, uses and releases one object per step without ever waiting.) */
int psattn_free_meta_async(psattn_meta* meta, void* hip_stream);

/* Frees every idle buffer pair of the pool (waits for the device to be done with
 * each).  Objects still alive are not touched. */
int psattn_trim_pool(void);

/* Host read-back of the canonical metadata (pure host copies, no synchronisation).
 * grid = PSATTN_GRID_FWD: rows are q-tiles, idx are k-tiles.
 * grid = PSATTN_GRID_BWD: rows are k-tiles, idx are q-tiles. */
int psattn_meta_tiles(const psattn_meta* meta, int32_t grid, int32_t* tile_q, int32_t* tile_k,
                      int32_t* n_q_tiles, int32_t* n_k_tiles, int64_t* n_entries);
int psattn_meta_copy_csr(const psattn_meta* meta, int32_t grid,
                         int32_t* row_ptr, /* host [n_rows + 1]                      */
                         int32_t* idx,     /* host [n_entries], ascending in a row   */
                         uint8_t* cls);    /* host [n_entries], PARTIAL or FULL      */
/* tok_desc: host [3 * T] = (s, hole_lo, hole_hi) per token. */
int psattn_meta_copy_tok_desc(const psattn_meta* meta, int32_t* tok_desc);
/* key_hi: host [T]; the queries allowed to read key j are exactly [j, key_hi[j])
 * (the end of the chosen response for chosen keys, else the end of the sample;
 * 0 for padding).  This is the mask seen from the key side, used by the dK/dV pass. */
int psattn_meta_copy_key_desc(const psattn_meta* meta, int32_t* key_hi);
/* Exact number of allowed (q, kv) pairs, from the closed form
 * sum_i tri(p) + sum_responses (len * p + tri(len)), tri(n) = n(n+1)/2
 * (two responses: tri(p) + c*p + tri(c) + r*p + tri(r)). */
int psattn_meta_allowed_pairs(const psattn_meta* meta, int64_t* n_allowed);

/*
 * First-Fit-Decreasing packing of samples into rows of row_len tokens (Section 4.3.2: an
 * FFD-based sampler packs each mini-batch; the packing length is batch size x maximum
 * sequence length and batches are padded to it).  The packing unit is a whole sample
 * (prompt + chosen + rejected): units are taken in order of decreasing length, equal
 * lengths in their original order, and each goes to the lowest-numbered row that still
 * has room, at the first free position of that row; a new row is opened only when no
 * open row has room.  Host only, integer only, O(n log n).
 *
 *   max_rows = 0: as many rows as needed.  max_rows > 0: at most that many rows (the
 *       fixed packing length of a mini-batch); a unit that fits nowhere gets offset -1.
 *   offset [n_samples] (host, out): flat start token of every sample, row * row_len +
 *       position in the row, in the caller's sample order; -1 = left out.
 *   order  [n_samples] (host, out): sample indices sorted by offset (left-out samples last).
 *       psattn_build_meta wants its sample table sorted by offset: pass offset[order[k]],
 *       prefix_len[order[k]], ... for the k placed samples, and total_tokens = *n_rows * row_len.
 *   n_rows, padding_tokens (host, out, may be NULL): rows opened; row capacity not covered
 *       by a placed sample.
 * Errors: PSATTN_EINVAL (null array, negative length, empty sample, row_len <= 0),
 * PSATTN_ERANGE (a sample longer than a row), PSATTN_EUNSUPPORTED (flat offsets would
 * not fit int32).
 */
int psattn_pack_ffd(int32_t n_samples, const int32_t* prefix_len, const int32_t* chosen_len,
                    const int32_t* rejected_len, int32_t row_len, int32_t max_rows,
                    int32_t* offset, int32_t* order, int32_t* n_rows, int64_t* padding_tokens);

/*
 * Forward: O = softmax(scale * Q K^T restricted to allowed pairs) V and
 * LSE[h, q] = log sum_kv exp(scale * Q_q . K_kv) (natural log).  SKIPPED tiles are
 * never computed (Section 3.1).  dt selects the element type of Q, K, V, O
 * (float, or bfloat16 with float accumulation); LSE is always float.
 * head_dim: 64 or 128 for either type.  The matrix-core kernels serve PSATTN_BF16 with
 * head_dim 128, scale > 0 and the default tile grids; every other valid request runs on
 * plain one-thread-per-row kernels that are orders of magnitude slower (they exist for the
 * fp32 correctness configuration).  psattn_uses_mfma tells which one a call would take.
 */
int psattn_fwd(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
               int32_t head_dim, float scale,
               const void* Q, const void* K, const void* V, /* device */
               void* O,                                     /* device [T, n_q_heads, head_dim] */
               float* LSE,                                  /* device [n_q_heads, T]           */
               void* hip_stream);

/*
 * Backward of psattn_fwd given dO, the forward's O and LSE: recomputes
 * P = exp(S - LSE), then dV = P^T dO, dS = P o (dO V^T - delta), delta = rowsum(dO o O),
 * dQ = scale dS K, dK = scale dS^T Q.  dK and dV of a kv-head sum over the G q-heads
 * that read it; prompt keys collect gradient from prompt, chosen and rejected
 * queries.  The paper times forward and backward together (Section 4.2).
 *
 * workspace: device scratch of at least psattn_bwd_workspace_bytes() bytes, owned by
 * the caller, contents undefined on entry and exit (holds delta and a rescaled copy of LSE).
 */
int psattn_bwd(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
               int32_t head_dim, float scale,
               const void* Q, const void* K, const void* V, const void* O, const void* dO,
               const float* LSE,                /* device, as written by psattn_fwd */
               void* dQ, void* dK, void* dV,    /* device, fully overwritten        */
               void* workspace, size_t workspace_bytes, void* hip_stream);

size_t psattn_bwd_workspace_bytes(const psattn_meta* meta, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim);

/*
 * psattn_bwd without a workspace argument, for callers that cannot allocate device
 * memory: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The scratch lives in a 32 MiB device array inside the library (one copy
 * per device, held until the process ends); the call allocates nothing.  Limit:
 * n_q_heads * T <= psattn_bwd_static_max_rows() (4 194 304), otherwise PSATTN_ELIMIT and
 * nothing is launched.  All calls on one device share that array: calls that overlap on
 * one device (different streams or threads) race; calls on one stream are safe.
 * Everything else is as for psattn_bwd.
 */
int psattn_bwd_static(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads,
                      int32_t head_dim, float scale,
                      const void* Q, const void* K, const void* V, const void* O, const void* dO,
                      const float* LSE, void* dQ, void* dK, void* dV, void* hip_stream);
size_t psattn_bwd_static_max_rows(void);

/* 1 if psattn_fwd (backward = 0) or psattn_bwd (backward != 0) would run the bf16
 * matrix-core kernels for this meta object, element type, head_dim and scale, 0 if
 * the call would run on the slow generic kernels, negative status for a NULL meta. */
int psattn_uses_mfma(const psattn_meta* meta, int32_t dt, int32_t head_dim, float scale, int32_t backward);

/*
 * Per-pass device timing for benchmarks.  While enabled, psattn_fwd / psattn_bwd
 * bracket each kernel with a pair of HIP events on the caller's stream (pass 0 =
 * forward, 1 = delta, 2 = dQ, 3 = dK/dV).  psattn_profile_read waits for the
 * recorded events, adds the elapsed milliseconds per pass to sum_ms[4] and the
 * number of launches to count[4] (both host, overwritten), and forgets them.
 * Not thread-safe; meant for one benchmarking thread.  At most 65 536 unread event
 * pairs are kept; launches beyond that are not timed until the next read.
 */
int psattn_profile_enable(int32_t on);
int psattn_profile_read(double* sum_ms, int64_t* count);

/*
 * Rotary position embedding inside the attention op, with the position ids of Section 3.1:
 * every response restarts right behind the prompt, so that each response sees the positions
 * it would have in the normal paired format (prompt tokens 0 .. p-1, the tokens of every
 * response p, p+1, ...; with psattn_build_meta_multi likewise for each of the k responses).
 * Convention: head dim i < head_dim/2 is paired with i + head_dim/2 and the pair is turned by
 * position * theta^(-2i/head_dim) ("rotate-half"); the result is rounded to bfloat16 like any
 * stored activation.  PSATTN_BF16 with head_dim 128 on the default tile grids only
 * (PSATTN_EUNSUPPORTED otherwise).
 *
 * psattn_rope_create builds the cos/sin table for positions [0, max_positions) on the current
 * device (host computes it in double precision; the call allocates device memory and waits
 * for its upload: create it once, not per step).  A meta object that needs more positions
 * than the table holds is refused with PSATTN_ELIMIT.
 *
 * psattn_fwd_rope: Q and K arrive UNROTATED.  K is rotated once into Kr (device
 * [T, n_kv_heads, 128], caller-owned), Q is rotated in registers as the forward loads it
 * and saved into Qr (device [T, n_q_heads, 128], caller-owned; NULL if no backward will
 * follow).  O and LSE as for psattn_fwd.  psattn_rope_k is the K half alone.
 *
 * psattn_bwd_rope: takes the forward's Qr and Kr; dQ and dK are the gradients with respect to
 * the UNROTATED Q and K (turned back in registers before they are stored), dV as usual.
 * Workspace as for psattn_bwd.
 *
 * psattn_meta_copy_positions: host read-back of the position id of every token (0 for
 * padding) and of the number of positions the object needs.
 */
int psattn_rope_create(int32_t head_dim, float theta, int32_t max_positions, void* hip_stream, psattn_rope** out);
int psattn_rope_free(psattn_rope* rope);
int psattn_rope_k(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_kv_heads, int32_t head_dim,
                  const void* K, void* Kr, void* hip_stream);
int psattn_fwd_rope(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_q_heads,
                    int32_t n_kv_heads, int32_t head_dim, float scale,
                    const void* Q, const void* K, const void* V, void* O, float* LSE,
                    void* Qr, void* Kr, void* hip_stream);
int psattn_bwd_rope(const psattn_meta* meta, const psattn_rope* rope, int32_t dt, int32_t n_q_heads,
                    int32_t n_kv_heads, int32_t head_dim, float scale,
                    const void* Qr, const void* Kr, const void* V, const void* O, const void* dO,
                    const float* LSE, void* dQ, void* dK, void* dV,
                    void* workspace, size_t workspace_bytes, void* hip_stream);
int psattn_meta_copy_positions(const psattn_meta* meta, int32_t* pos /* host [T] */, int32_t* n_positions);

/*
 * Per-response log-probabilities and the DPO loss (Section 2.1, Eq. 1: the loss needs
 * log pi(y | x), the total log-probability of each completion).  In the prefix-shared
 * sequence the logits row of a token predicts the next token of the token's own branch:
 * inside a response the following token; the LAST prompt token predicts the first token of
 * every response.  Other prompt rows, the last row of every response and padding predict
 * nothing and are never read.  A response behind an empty prompt has nothing to predict its
 * first token from; that token contributes nothing.
 *
 * psattn_logprob_plan: from the sample table (host arrays, as for psattn_build_meta_multi;
 * the paper's format is two responses per sample, chosen then rejected) builds the small
 * device tables the passes need.  Allocates device memory and waits for its upload.
 *
 * psattn_logprob_fwd: logits device [T, vocab] (float or bfloat16 by dt), token_ids device
 * int32 [T].  Writes row_lse[t] = log sum exp(logits[t, :]) for every row that predicts
 * something (device float [T]; other entries untouched) and resp_logp[j] = log pi(response j
 * | prompt) (device float [n_responses]), fp32 accumulation in a fixed order.
 *
 * A token id outside [0, vocab) contributes nothing to its response (and nothing is read or
 * written for it).
 *
 * psattn_logprob_bwd: dlogits (device [T, vocab], dt; fully overwritten) = gradient of
 * sum_j d_resp_logp[j] * resp_logp[j]: every predicting row gets, per item, d_resp_logp[j] *
 * (onehot(target) - softmax(row)); rows that predict nothing are written as zeros.
 *
 * psattn_dpo_loss: responses stored as (chosen, rejected) pairs: loss[i] = -log sigmoid(beta *
 * ((pc - rc) - (pr - rr))) from policy and reference log-probabilities (device float
 * [2 n_pairs] each); d_logp (device float [2 n_pairs], may be NULL) = d loss[i] / d policy
 * log-probabilities.  (Eq. 1 is printed with a ratio of logarithms; it is read with the
 * logarithm of the ratio, as DPO is defined.)
 */
int psattn_logprob_plan(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                        const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                        void* hip_stream, psattn_lp_plan** out);
int psattn_logprob_plan_free(psattn_lp_plan* plan);
int psattn_logprob_plan_info(const psattn_lp_plan* plan, int32_t* n_responses, int32_t* n_rows, int64_t* n_items);
int psattn_logprob_fwd(const psattn_lp_plan* plan, int32_t dt, int32_t vocab, const void* logits,
                       const int32_t* token_ids, float* row_lse, float* resp_logp, void* hip_stream);
int psattn_logprob_bwd(const psattn_lp_plan* plan, int32_t dt, int32_t vocab, const void* logits,
                       const int32_t* token_ids, const float* row_lse, const float* d_resp_logp,
                       void* dlogits, void* hip_stream);
int psattn_dpo_loss(int32_t n_pairs, float beta, const float* logp_policy, const float* logp_ref,
                    float* loss, float* d_logp, void* hip_stream);

/*
 * Measurement aid (no part of the computation): issues the memory operations that a
 * one-pass backward would add for dQ, and nothing else.  One workgroup per (k-tile,
 * kv-head) walks the k-major tile list of the default grid and adds (mode 0: fp32 atomic
 * add, mode 1: plain store) a 64 x 128 fp32 tile into acc [T, n_q_heads, 128] (device)
 * for every (q-tile, q-head) it visits.  Timing it against the separate dQ pass decides
 * between the two backward designs.  acc is modified.
 */
int psattn_probe_dq_atomics(const psattn_meta* meta, int32_t n_q_heads, int32_t n_kv_heads, float* acc,
                            int32_t mode, void* hip_stream);

/*
 * Measurement aid: the matrix-core ceiling.  Launches n_workgroups workgroups of 4 waves that each
 * issue 4 * iters (iters even) back-to-back v_mfma_f32_32x32x16_bf16 (32 768 FLOPs each per wave) on
 * register operands, with no memory traffic; sink is one device float that is never written.  FLOPs
 * launched = n_workgroups * 4 * 4 * iters * 32768.  random_operands = 0: one constant fragment per
 * operand side; 1: eight fragments per side with random sign and mantissa bits (magnitudes 0.5 to
 * 2), a different pair on every MFMA (the clock the device holds under matrix load depends on how
 * much the data toggles); 2: the eight-fragment register pattern of 1 holding the constants of 0.
 */
int psattn_probe_mfma_peak(int32_t n_workgroups, int32_t iters, int32_t random_operands, float* sink,
                           void* hip_stream);

/* Name of the kernel that psattn_fwd / psattn_bwd launched most recently in this
 * process for the given pass (0 = forward, 1 = delta, 2 = dQ, 3 = dK/dV), for profilers
 * and benchmarks; before any launch of that pass, the kernel a default-grid call with
 * element type dt would use. */
const char* psattn_kernel_name(int32_t dt, int32_t pass);

const char* psattn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PSATTN_H */
