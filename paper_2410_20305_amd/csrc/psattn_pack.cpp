// Host packer: First-Fit-Decreasing placement of samples into fixed-length rows
// (Section 4.3.2: an FFD-based sampler packs the mini-batch; the packing length is
// batch size x maximum sequence length and every batch is padded to it).  The unit of
// packing is a whole sample, prompt + chosen + rejected (Section 3.2: the two responses
// of a sample cannot be packed independently).  Integer only.
//
// First fit over many rows is answered by a max-tree over the rows' free space: the
// first row with enough room is found by descending from the root, O(log rows) per
// unit instead of a scan.
#include <algorithm>
#include <cstdint>
#include <new>
#include <numeric>
#include <vector>

#include "psattn.h"

namespace {

// leaves = free tokens per row; inner node = max of its children
struct FreeTree {
    int32_t leaves = 1;
    std::vector<int32_t> node;
    explicit FreeTree(int32_t n_rows, int32_t row_len) {
        while (leaves < n_rows) leaves *= 2;
        node.assign(2 * static_cast<size_t>(leaves), 0);
        for (int32_t i = 0; i < n_rows; ++i) node[leaves + i] = row_len;
        for (int32_t i = leaves - 1; i >= 1; --i) node[i] = std::max(node[2 * i], node[2 * i + 1]);
    }
    // lowest row index with at least `need` free tokens, -1 if none
    int32_t first_fit(int32_t need) const {
        if (node[1] < need) return -1;
        int32_t i = 1;
        while (i < leaves) i = node[2 * i] >= need ? 2 * i : 2 * i + 1;
        return i - leaves;
    }
    int32_t free_of(int32_t row) const { return node[leaves + row]; }
    void take(int32_t row, int32_t n) {
        int32_t i = leaves + row;
        node[i] -= n;
        for (i /= 2; i >= 1; i /= 2) node[i] = std::max(node[2 * i], node[2 * i + 1]);
    }
};

}  // namespace

extern "C" int psattn_pack_ffd(int32_t n_samples, const int32_t* prefix_len, const int32_t* chosen_len,
                               const int32_t* rejected_len, int32_t row_len, int32_t max_rows, int32_t* offset,
                               int32_t* order, int32_t* n_rows, int64_t* padding_tokens) {
    if (n_samples < 0 || row_len <= 0 || max_rows < 0) return PSATTN_EINVAL;
    if (n_samples > 0 && (!prefix_len || !chosen_len || !rejected_len || !offset || !order)) return PSATTN_EINVAL;
    try {
        std::vector<int64_t> len(n_samples);
        for (int32_t i = 0; i < n_samples; ++i) {
            if (prefix_len[i] < 0 || chosen_len[i] < 0 || rejected_len[i] < 0) return PSATTN_EINVAL;
            len[i] = static_cast<int64_t>(prefix_len[i]) + chosen_len[i] + rejected_len[i];
            if (len[i] == 0) return PSATTN_EINVAL;
            if (len[i] > row_len) return PSATTN_ERANGE;
        }
        // decreasing length, equal lengths in their original order
        std::vector<int32_t> by_len(n_samples);
        std::iota(by_len.begin(), by_len.end(), 0);
        std::stable_sort(by_len.begin(), by_len.end(), [&](int32_t a, int32_t b) { return len[a] > len[b]; });
        // Rows that can ever be opened: one per unit at most, and first fit leaves at most one
        // row no more than half full, so also no more than 2 * total / row_len + 1.
        int64_t total = 0;
        for (int64_t l : len) total += l;
        int64_t cap64 = std::min<int64_t>(std::max(n_samples, 1), 2 * total / row_len + 1);
        if (max_rows > 0) cap64 = std::min<int64_t>(cap64, max_rows);
        if (cap64 * row_len > INT32_MAX) return PSATTN_EUNSUPPORTED;  // flat offsets are int32
        const int32_t cap = static_cast<int32_t>(std::max<int64_t>(cap64, 1));
        FreeTree tree(cap, row_len);
        int32_t opened = 0;
        for (int32_t i : by_len) {
            const int32_t need = static_cast<int32_t>(len[i]);
            const int32_t r = tree.first_fit(need);
            if (r < 0) {  // only with max_rows > 0: the unit is left out
                offset[i] = -1;
                continue;
            }
            offset[i] = static_cast<int32_t>(static_cast<int64_t>(r) * row_len + (row_len - tree.free_of(r)));
            tree.take(r, need);
            opened = std::max(opened, r + 1);
        }
        // buffer order: by offset; units that were left out go last, in their original order
        std::iota(order, order + n_samples, 0);
        std::stable_sort(order, order + n_samples, [&](int32_t a, int32_t b) {
            const uint32_t x = static_cast<uint32_t>(offset[a]), y = static_cast<uint32_t>(offset[b]);  // -1 -> largest
            return x < y;
        });
        if (n_rows) *n_rows = opened;
        if (padding_tokens) {
            int64_t used = 0;
            for (int32_t i = 0; i < n_samples; ++i)
                if (offset[i] >= 0) used += len[i];
            *padding_tokens = static_cast<int64_t>(opened) * row_len - used;
        }
    } catch (const std::bad_alloc&) {
        return PSATTN_ENOMEM;
    }
    return PSATTN_OK;
}
