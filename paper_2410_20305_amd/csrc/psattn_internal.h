// Internal declarations shared by the host metadata builder, the C-ABI entry
// points and the kernel launchers of libpsattn.  Not part of the public ABI.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "psattn.h"

namespace psattn {

constexpr int32_t kPadStart = INT32_MAX;

// Default tile grids = the shapes the bf16 MFMA kernels are built for.
constexpr int32_t kFwdTileQ = 128;
constexpr int32_t kFwdTileK = 64;
constexpr int32_t kBwdTileQ = 64;
constexpr int32_t kBwdTileK = 128;

// One CSR over a tile grid.  entry = (column tile index << 2) | class.
struct TileCsr {
    int32_t tile_q = 0, tile_k = 0;
    int32_t n_q_tiles = 0, n_k_tiles = 0;
    std::vector<int32_t> row_ptr;  // rows = q-tiles (FWD) or k-tiles (BWD)
    std::vector<int32_t> idx;
    std::vector<uint8_t> cls;
    std::vector<int32_t> order;    // rows sorted by decreasing work (longest first)
};

// What a workgroup of the MFMA kernels needs to start on its row, in launch order: one
// 16-byte scalar load instead of a chain of three dependent ones (launch order -> row ->
// list bounds -> first entry), which is a noticeable part of a short workgroup's life.
struct alignas(16) RowLaunch {
    int32_t row;          // tile row (q-tile for the q-major grid, k-tile for the k-major one)
    int32_t begin;        // first position of the row's tile list in `entry`
    int32_t count;        // its length
    int32_t first_entry;  // the entry the walk starts with: entry[begin] for the q-major grid,
                          // entry[begin + count - 1] for the k-major one (walked backwards)
};

// Device-side view handed to kernels by value.
struct DeviceCsr {
    const int32_t* row_ptr;
    const int32_t* entry;  // (idx << 2) | cls
    const int32_t* order;
    const RowLaunch* launch;  // [n_rows], in launch order
    int32_t n_rows;
    int32_t tile_q, tile_k;
};

// Per-token descriptor as the kernels read it (one 16-byte load).
struct alignas(16) Tok4 {
    int32_t s, hole_lo, hole_hi, key_hi;
};

struct DeviceMeta {
    const Tok4* tok;        // [T]
    DeviceCsr fwd, bwd;
    int32_t T;
};

}  // namespace psattn

struct psattn_meta {
    int32_t T = 0;
    int32_t n_samples = 0;
    int64_t n_allowed = 0;
    int32_t n_positions = 0;        // 1 + the largest position id of any token (prompt length + longest response)
    std::vector<int32_t> tok_desc;  // [3T]  (s, hole_lo, hole_hi)
    std::vector<int32_t> key_hi;    // [T]   queries that may read key j are [j, key_hi[j])
    psattn::TileCsr fwd, bwd;
    // device copy
    bool on_device = false;
    int device = -1;
    void* d_blob = nullptr;   // device copy of the metadata (from the library's blob pool)
    void* h_stage = nullptr;  // pinned staging buffer of the same size, alive until release
    size_t blob_bytes = 0;    // bytes in use
    size_t blob_cap = 0;      // bytes allocated
    void* blob_idle = nullptr;  // hipEvent_t of the pooled pair
    psattn::DeviceMeta dev{};
};

namespace psattn {

// Host-only construction (psattn_meta.cpp).  Returns a psattn_status.
int build_host(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
               const int32_t* chosen_len, const int32_t* rejected_len, int32_t total_tokens,
               int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
               psattn_meta** out);

int build_host_multi(int32_t n_samples, const int32_t* offset, const int32_t* prefix_len,
                     const int32_t* resp_ptr, const int32_t* resp_len, int32_t total_tokens,
                     int32_t tile_q, int32_t tile_k, int32_t bwd_tile_q, int32_t bwd_tile_k,
                     psattn_meta** out);

struct AttnArgs {
    DeviceMeta meta;
    int32_t Hq, Hkv, d;
    float scale;
    const void *Q, *K, *V, *O, *dO;
    const float* LSE;
    void *Oout, *dQ, *dK, *dV;
    float* LSEout;
    // Rotary embedding (nullptr = none): table [positions][128] = cos[64] | sin[64] per position id.
    // Forward: Q arrives unrotated, is rotated in registers and, if Qr is set, saved rotated for the
    // backward; K arrives rotated.  Backward: Q and K arrive rotated, dQ and dK leave unrotated.
    const float* rope;
    void* Qr;
    float* delta;  // [Hq, T]  workspace: rowsum(dO o O); the MFMA kernels keep its negative here
    float* lse2;   // [Hq, T]  workspace: LSE * log2(e), written by the MFMA dQ pass for the dK/dV pass
};

// psattn_fwd with optional rotary embedding (rope_table == nullptr: none).
int fwd_checked(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                float scale, const void* Q, const void* K, const void* V, void* O, float* LSE,
                const float* rope_table, void* Qr, void* hip_stream);

// psattn_bwd without the workspace-size lookup: argument checks, then delta / dQ / dK/dV
// on `scratch_base` (device memory of at least bwd_scratch_bytes()).  Returns a psattn_status.
size_t bwd_scratch_bytes(const psattn_meta* meta, int32_t n_q_heads);
int bwd_checked(const psattn_meta* meta, int32_t dt, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                float scale, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                const float* LSE, void* dQ, void* dK, void* dV, void* scratch_base, size_t scratch_bytes,
                void* hip_stream, const float* rope_table = nullptr);

// Launchers (each returns a hipError_t cast to int; 0 = success).
int launch_generic_fwd(int dt, const AttnArgs& a, void* stream);
int launch_generic_dq(int dt, const AttnArgs& a, void* stream);
int launch_generic_dkdv(int dt, const AttnArgs& a, void* stream);
int launch_delta(int dt, const AttnArgs& a, void* stream);
int launch_mfma_fwd(const AttnArgs& a, void* stream);
int launch_mfma_dq(const AttnArgs& a, void* stream);
int launch_mfma_dkdv(const AttnArgs& a, void* stream);

}  // namespace psattn
