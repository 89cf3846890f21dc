// Host-side tile schedule of the Markovian next-scale mask (paper Sec. "Efficient Markovian
// Next-Scale Prediction", Eq. 4; appendix "Attention Patterns").
//
// From the prefix sums of the scale sizes the builder derives, for each direction, the
// list of workgroup items the kernels walk.  An item owns a contiguous range of rows of
// the stationary operand and visits one contiguous range of rows of the streamed
// operand; score tiles outside that range are never loaded.
//   direction 0 (forward, dQ): owned rows are queries, visited rows are keys.
//       Markovian mask:    query i of scale k (0-based) pairs with keys [off[max(k-1,0)], off[k+1])
//       block-causal mask: (VAR, paper Sec. "Background") with keys [0, off[k+1])
//   direction 1 (dK/dV): owned rows are keys, visited rows are queries.
//       Markovian mask:    key j of scale k pairs with queries [off[k], off[min(k+2,K)])
//       block-causal mask: with queries [off[k], L)
// (Inference steps need no tables: every query row of a step pairs with every key row.)
#pragma once
#include <cstdint>
#include <vector>

namespace hmar {

struct TileItem {
    int32_t own_begin, own_end;      // rows owned by the workgroup, own_end - own_begin <= rows_per_item
    int32_t other_begin, other_end;  // union of the owned rows' pair ranges
};

enum MaskKind : int32_t { kMaskMarkov = 0, kMaskBlockCausal = 1 };

struct Schedule {
    std::vector<int32_t> sides;      // as given: side lengths or token counts
    bool sizes_are_counts = false;   // the entries of `sides` are token counts n_k, not side lengths
    int32_t mask_kind = kMaskMarkov;
    std::vector<int32_t> off;        // K+1 prefix sums of the token counts n_k
    int32_t L = 0;                   // rows of Q, O, LSE per head
    int32_t Lk = 0;                  // rows of K, V per head (= L)
    int64_t allowed_pairs = 0;       // sum_k n_k (n_{k-1} + n_k)
    // per direction
    std::vector<TileItem> items[2];
    std::vector<int32_t> row_lo[2], row_hi[2];   // L entries each
};

// sizes: per scale the side length s_k (n_k = s_k^2 tokens, square token maps) or, with
// sizes_are_counts, the token count n_k itself (the paper's scales are H_k x W_k maps, Sec.
// "Background").
// rows_per_item: most rows one workgroup owns (a multiple of 32).  Returns false when the
// sizes are invalid (non-positive, too many, or L beyond max_len).
bool build_schedule(const int32_t* sizes, int32_t num_scales, bool sizes_are_counts, int32_t mask_kind,
                    int32_t rows_per_item, int32_t max_scales, int64_t max_len, Schedule* out);

}  // namespace hmar
