// Tile-schedule builder: pure host code, no HIP.  See schedule.h.
#include "schedule.h"

#include <algorithm>

namespace hmar {

static void partition_rows(const Schedule& s, int32_t rows_per_item, std::vector<TileItem>* items) {
    const int K = (int)s.sides.size();
    int32_t pend_begin = 0, pend_rows = 0;
    auto flush = [&]() {
        if (pend_rows > 0) items->push_back({pend_begin, pend_begin + pend_rows, 0, 0});
        pend_begin += pend_rows;
        pend_rows = 0;
    };
    for (int k = 0; k < K; ++k) {
        const int32_t n = s.off[k + 1] - s.off[k];
        if (2 * n >= rows_per_item) {
            // a scale big enough to fill workgroups on its own: split it into equal chunks,
            // each a multiple of 32 rows (one wavefront owns 32 rows) except the last
            flush();
            const int32_t chunks = (n + rows_per_item - 1) / rows_per_item;
            int32_t per = (n + chunks - 1) / chunks;
            per = (per + 31) / 32 * 32;
            for (int32_t b = s.off[k]; b < s.off[k + 1]; b += per)
                items->push_back({b, std::min(b + per, s.off[k + 1]), 0, 0});
            pend_begin = s.off[k + 1];
        } else {
            // small scales share a workgroup; their rows carry their own pair ranges
            if (pend_rows + n > rows_per_item) flush();
            pend_rows += n;
        }
    }
    flush();
}

bool build_schedule(const int32_t* sides, int32_t num_scales, bool sizes_are_counts, int32_t mask_kind,
                    int32_t rows_per_item, int32_t max_scales, int64_t max_len, Schedule* out) {
    if (!sides || num_scales < 1 || num_scales > max_scales || rows_per_item < 32 || rows_per_item % 32) return false;
    if (mask_kind != kMaskMarkov && mask_kind != kMaskBlockCausal) return false;
    Schedule s;
    s.mask_kind = mask_kind;
    s.sizes_are_counts = sizes_are_counts;
    s.sides.assign(sides, sides + num_scales);
    s.off.assign(1, 0);
    int64_t L = 0;
    for (int k = 0; k < num_scales; ++k) {
        if (sides[k] < 1 || (!sizes_are_counts && sides[k] > 46340)) return false;
        L += sizes_are_counts ? (int64_t)sides[k] : (int64_t)sides[k] * sides[k];
        if (L > max_len) return false;
        s.off.push_back((int32_t)L);
    }
    s.L = s.Lk = (int32_t)L;
    const int K = num_scales;
    const bool causal = mask_kind == kMaskBlockCausal;
    s.allowed_pairs = 0;
    for (int k = 0; k < K; ++k) {
        const int64_t n = s.off[k + 1] - s.off[k];
        const int64_t np = causal ? s.off[k] : (k > 0 ? s.off[k] - s.off[k - 1] : 0);
        s.allowed_pairs += n * (np + n);
    }
    for (int dir = 0; dir < 2; ++dir) {
        s.row_lo[dir].resize(s.L);
        s.row_hi[dir].resize(s.L);
        for (int k = 0; k < K; ++k) {
            int32_t lo, hi;
            if (dir == 0) { lo = causal ? 0 : s.off[std::max(k - 1, 0)]; hi = s.off[k + 1]; }
            else          { lo = s.off[k]; hi = causal ? s.L : s.off[std::min(k + 2, K)]; }
            for (int32_t r = s.off[k]; r < s.off[k + 1]; ++r) { s.row_lo[dir][r] = lo; s.row_hi[dir][r] = hi; }
        }
        partition_rows(s, rows_per_item, &s.items[dir]);
        for (TileItem& it : s.items[dir]) {
            int32_t lo = s.L, hi = 0;
            for (int32_t r = it.own_begin; r < it.own_end; ++r) {
                lo = std::min(lo, s.row_lo[dir][r]);
                hi = std::max(hi, s.row_hi[dir][r]);
            }
            it.other_begin = lo;
            it.other_end = hi;
        }
        // heaviest items first: the light ones fill the tail of the launch
        std::stable_sort(s.items[dir].begin(), s.items[dir].end(), [](const TileItem& a, const TileItem& b) {
            const int64_t ca = (int64_t)(a.own_end - a.own_begin) * (a.other_end - a.other_begin);
            const int64_t cb = (int64_t)(b.own_end - b.own_begin) * (b.other_end - b.other_begin);
            return ca > cb;
        });
    }
    *out = std::move(s);
    return true;
}

}  // namespace hmar
