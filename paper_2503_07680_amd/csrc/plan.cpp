// Host-side planner of one pack: greedy in-order fill -> cu_seqlens, then the tile worklist
// sorted by exact causal cost, longest first (Attention Balance Sort, paper Algorithm 7,
// applied to (sample, tile) work items instead of packs; pack cost a = sum len^2).
#include "hbp.h"

#include <algorithm>
#include <numeric>
#include <new>
#include <vector>

namespace {

struct Item {
  int64_t cost;
  hbp_tile t;
};

// pairs (r,k), 0 <= k <= r, with the in-sample query index r in [lo,hi): sum_{r}(r+1)
inline int64_t query_tile_pairs(int64_t lo, int64_t hi) {
  return (hi * (hi + 1) - lo * (lo + 1)) / 2;
}
// pairs with the in-sample key index k in [lo,hi) of a sample of s rows: sum_{k}(s-k)
inline int64_t key_tile_pairs(int64_t lo, int64_t hi, int64_t s) {
  const int64_t n = hi - lo;
  return n * s - (lo + hi - 1) * n / 2;
}

}  // namespace

static hbp_status hbp_pack_plan_impl(const int32_t* lengths, int32_t n_lengths, int32_t pack_len,
                                    int32_t tile_rows, int32_t kind, int32_t* cu_seqlens,
                                    int32_t cu_cap, int32_t* n_samples_out,
                                    int32_t* n_consumed_out, hbp_tile* tiles, int64_t* tile_cost,
                                    int32_t tile_cap, int32_t* n_tiles_out,
                                    int64_t* pack_cost_out) {
  if (!n_samples_out || !n_consumed_out || !n_tiles_out || !pack_cost_out)
    return HBP_ERR_INVALID_ARG;
  *n_samples_out = *n_consumed_out = *n_tiles_out = 0;
  *pack_cost_out = 0;
  if (n_lengths < 0 || (n_lengths > 0 && !lengths)) return HBP_ERR_INVALID_ARG;
  if (pack_len <= 0 || tile_rows <= 0) return HBP_ERR_INVALID_ARG;
  if (kind != HBP_TILES_QUERY && kind != HBP_TILES_KEY) return HBP_ERR_INVALID_ARG;
  if (cu_cap < 0 || tile_cap < 0) return HBP_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_lengths; ++i)
    if (lengths[i] <= 0) return HBP_ERR_INVALID_ARG;

  // Packing: in-order fill, last sample truncated to the space that is left.
  std::vector<int32_t> cu(1, 0);
  int32_t consumed = 0;
  for (int32_t i = 0; i < n_lengths && cu.back() < pack_len; ++i) {
    const int32_t room = pack_len - cu.back();
    cu.push_back(cu.back() + std::min(lengths[i], room));
    ++consumed;
  }
  const int32_t n = static_cast<int32_t>(cu.size()) - 1;

  int64_t pack_cost = 0;
  std::vector<Item> items;
  for (int32_t i = 0; i < n; ++i) {
    const int64_t s = cu[i + 1] - cu[i];
    pack_cost += s * s;
    int32_t t = 0;
    for (int64_t lo = 0; lo < s; lo += tile_rows, ++t) {
      const int64_t hi = std::min<int64_t>(lo + tile_rows, s);
      Item it;
      it.cost = kind == HBP_TILES_QUERY ? query_tile_pairs(lo, hi) : key_tile_pairs(lo, hi, s);
      it.t.sample = i;
      it.t.tile = t;
      it.t.row_begin = cu[i] + static_cast<int32_t>(lo);
      it.t.row_end = cu[i] + static_cast<int32_t>(hi);
      items.push_back(it);
    }
  }
  std::sort(items.begin(), items.end(), [](const Item& a, const Item& b) {
    if (a.cost != b.cost) return a.cost > b.cost;
    if (a.t.sample != b.t.sample) return a.t.sample < b.t.sample;
    return a.t.tile < b.t.tile;
  });

  *n_samples_out = n;
  *n_consumed_out = consumed;
  *n_tiles_out = static_cast<int32_t>(items.size());
  *pack_cost_out = pack_cost;

  hbp_status st = HBP_OK;
  if (cu_seqlens) {
    if (cu_cap < n + 1) {
      st = HBP_ERR_CAPACITY;
    } else {
      std::copy(cu.begin(), cu.end(), cu_seqlens);
    }
  }
  if (tiles || tile_cost) {
    if (tile_cap < static_cast<int32_t>(items.size())) {
      st = HBP_ERR_CAPACITY;
    } else {
      for (size_t j = 0; j < items.size(); ++j) {
        if (tiles) tiles[j] = items[j].t;
        if (tile_cost) tile_cost[j] = items[j].cost;
      }
    }
  }
  return st;
}

// The planner allocates host memory: running out of it is reported, never thrown across the C boundary.
extern "C" hbp_status hbp_pack_plan(const int32_t* lengths, int32_t n_lengths, int32_t pack_len,
                                    int32_t tile_rows, int32_t kind, int32_t* cu_seqlens,
                                    int32_t cu_cap, int32_t* n_samples_out,
                                    int32_t* n_consumed_out, hbp_tile* tiles, int64_t* tile_cost,
                                    int32_t tile_cap, int32_t* n_tiles_out,
                                    int64_t* pack_cost_out) {
  try {
    return hbp_pack_plan_impl(lengths, n_lengths, pack_len, tile_rows, kind, cu_seqlens, cu_cap, n_samples_out, n_consumed_out,
                              tiles, tile_cost, tile_cap, n_tiles_out, pack_cost_out);
  } catch (const std::bad_alloc&) {
    return HBP_ERR_NO_MEMORY;
  } catch (...) {
    return HBP_ERR_INVALID_ARG;
  }
}
