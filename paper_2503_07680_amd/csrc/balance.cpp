// Host-side multi-level Balance Packing planner (paper Section 4.2, Algorithm 2; appendix functions
// GroupData, GreedyFill, Attention Balance Sort; metrics of Section 3.1).  Integer arithmetic only.
//
// The paper's procedures are stated as nested scans over lists; the results here are the same as
// those scans would give, found with two small search trees so that a million samples take well
// under a second:
//   * first-fit (Packing): "the first pack, in creation order, with room for x" is the leftmost
//     leaf >= len(x) of a max-tree over the packs' free space (unopened packs count as empty);
//   * GreedyFill: "the next x of D_j, in order, that still fits" is the leftmost leaf <= room at or
//     after the scan position of a min-tree over the lengths of the samples still in D_j.
#include "hbp.h"

#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

namespace {

constexpr int32_t kGone = std::numeric_limits<int32_t>::max();

// complete binary tree over n leaves; node value = min (or max) of its leaves
template <bool IS_MIN>
class LeafTree {
 public:
  LeafTree(const std::vector<int32_t>& leaves) {
    n_ = 1;
    while (n_ < (int64_t)leaves.size()) n_ <<= 1;
    t_.assign(2 * n_, IS_MIN ? kGone : -1);
    for (size_t i = 0; i < leaves.size(); ++i) t_[n_ + i] = leaves[i];
    for (int64_t i = n_ - 1; i >= 1; --i) t_[i] = pick(t_[2 * i], t_[2 * i + 1]);
  }
  void set(int64_t leaf, int32_t v) {
    int64_t i = n_ + leaf;
    t_[i] = v;
    for (i >>= 1; i >= 1; i >>= 1) t_[i] = pick(t_[2 * i], t_[2 * i + 1]);
  }
  int32_t get(int64_t leaf) const { return t_[n_ + leaf]; }
  // leftmost leaf at index >= from whose value is <= bound (min tree) / >= bound (max tree); -1 if none
  int64_t leftmost(int64_t from, int32_t bound) const {
    if (from >= n_) return -1;
    return descend(1, 0, n_, from, bound);
  }

 private:
  static int32_t pick(int32_t a, int32_t b) { return IS_MIN ? std::min(a, b) : std::max(a, b); }
  static bool ok(int32_t v, int32_t bound) { return IS_MIN ? v <= bound : v >= bound; }
  int64_t descend(int64_t node, int64_t lo, int64_t hi, int64_t from, int32_t bound) const {
    if (hi <= from || !ok(t_[node], bound)) return -1;
    if (hi - lo == 1) return lo;
    const int64_t mid = (lo + hi) / 2;
    const int64_t l = descend(2 * node, lo, mid, from, bound);
    return l >= 0 ? l : descend(2 * node + 1, mid, hi, from, bound);
  }
  int64_t n_;
  std::vector<int32_t> t_;
};

struct Pack {
  std::vector<int32_t> items;
  int32_t tokens = 0;
  int64_t attn = 0;
};

// splitmix64 (Steele, Lea, Flood 2014)
struct SplitMix64 {
  uint64_t s;
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
};

double ratio_to_max(const std::vector<int64_t>& v) {
  const int64_t m = *std::max_element(v.begin(), v.end());
  if (m == 0) return 0.0;
  double s = 0.0;
  for (int64_t x : v) s += (double)(m - x);
  return s / ((double)m * (double)v.size());
}

}  // namespace

static hbp_status hbp_balance_packing_impl(const int32_t* lengths, int32_t n_samples,
                                          const int32_t* group_lens, const int32_t* packs_per_batch,
                                          const int32_t* level_sp, int32_t n_levels,
                                          uint64_t shuffle_seed, int32_t* pack_items, int32_t item_cap,
                                          hbp_pack* packs, int32_t pack_cap, int32_t* n_packs_out,
                                          hbp_batch* batches, int32_t batch_cap, int32_t* n_batches_out,
                                          hbp_pack_metrics* metrics_or_null) {
  if (!n_packs_out || !n_batches_out) return HBP_ERR_INVALID_ARG;
  *n_packs_out = *n_batches_out = 0;
  if (n_samples < 0 || (n_samples > 0 && !lengths)) return HBP_ERR_INVALID_ARG;
  if (n_levels < 1 || !group_lens || !packs_per_batch) return HBP_ERR_INVALID_ARG;
  if (item_cap < 0 || pack_cap < 0 || batch_cap < 0) return HBP_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_levels; ++i) {
    if (group_lens[i] <= (i ? group_lens[i - 1] : 0) || packs_per_batch[i] <= 0) return HBP_ERR_INVALID_ARG;
    if (level_sp && level_sp[i] < 1) return HBP_ERR_INVALID_ARG;
  }
  for (int32_t x = 0; x < n_samples; ++x)
    if (lengths[x] <= 0 || lengths[x] > group_lens[n_levels - 1]) return HBP_ERR_INVALID_ARG;

  // GroupData: D_i = samples with length in (l_{i-1}, l_i], input order
  std::vector<std::vector<int32_t>> d(n_levels);
  for (int32_t x = 0; x < n_samples; ++x) {
    const int32_t i = (int32_t)(std::lower_bound(group_lens, group_lens + n_levels, lengths[x]) - group_lens);
    d[i].push_back(x);
  }
  // what is still in D_j: a min-tree over the lengths in list order, kGone once taken
  std::vector<LeafTree<true>> left;
  left.reserve(n_levels);
  for (int32_t i = 0; i < n_levels; ++i) {
    std::vector<int32_t> len(d[i].size());
    for (size_t k = 0; k < d[i].size(); ++k) len[k] = lengths[d[i][k]];
    left.emplace_back(len);
  }

  std::vector<Pack> all_packs;
  std::vector<hbp_batch> all_batches;
  for (int32_t i = n_levels - 1; i >= 0; --i) {
    const int32_t cap = group_lens[i];
    // Packing(D_i, l_i): first-fit decreasing over what GreedyFill of the larger groups left in D_i
    std::vector<int32_t> mine;
    for (size_t k = 0; k < d[i].size(); ++k)
      if (left[i].get((int64_t)k) != kGone) mine.push_back(d[i][k]);
    std::stable_sort(mine.begin(), mine.end(), [&](int32_t a, int32_t b) { return lengths[a] > lengths[b]; });
    std::vector<Pack> g;
    {
      LeafTree<false> room(std::vector<int32_t>(mine.size(), cap));
      for (int32_t x : mine) {
        const int64_t p = room.leftmost(0, lengths[x]);  // exists: an unopened pack has room for any x <= cap
        if ((size_t)p == g.size()) g.emplace_back();
        g[p].items.push_back(x);
        g[p].tokens += lengths[x];
        room.set(p, cap - g[p].tokens);
      }
    }
    // GreedyFill(G_i, l_i, [D_{i-1}, ..., D_1])
    for (Pack& pk : g) {
      for (int32_t j = i - 1; j >= 0 && pk.tokens < cap; --j) {
        int64_t pos = 0;
        for (;;) {
          const int64_t k = left[j].leftmost(pos, cap - pk.tokens);
          if (k < 0) break;
          const int32_t x = d[j][k];
          pk.items.push_back(x);
          pk.tokens += lengths[x];
          left[j].set(k, kGone);
          pos = k + 1;
        }
      }
    }
    // Attention Balance Sort: a = sum len^2, descending, ties by creation order; then mini-batches
    for (Pack& pk : g) {
      pk.attn = 0;
      for (int32_t x : pk.items) pk.attn += (int64_t)lengths[x] * lengths[x];
    }
    std::vector<int32_t> order(g.size());
    for (size_t k = 0; k < g.size(); ++k) order[k] = (int32_t)k;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return g[a].attn > g[b].attn; });
    for (size_t k = 0; k < order.size(); ++k) {
      if (k % (size_t)packs_per_batch[i] == 0) all_batches.push_back(hbp_batch{i, (int32_t)all_packs.size(), 0, 0});
      ++all_batches.back().n_packs;
      all_packs.push_back(std::move(g[order[k]]));
    }
  }
  // Shuffle(B): Fisher-Yates from the end, j = next() mod (k + 1)
  SplitMix64 rng{shuffle_seed};
  for (int64_t k = (int64_t)all_batches.size() - 1; k >= 1; --k) {
    const int64_t j = (int64_t)(rng.next() % (uint64_t)(k + 1));
    std::swap(all_batches[k], all_batches[j]);
  }

  *n_packs_out = (int32_t)all_packs.size();
  *n_batches_out = (int32_t)all_batches.size();
  const bool want_lists = pack_items || packs || batches;
  if (want_lists) {
    if (!pack_items || !packs || !batches) return HBP_ERR_INVALID_ARG;
    if (item_cap < n_samples || pack_cap < *n_packs_out || batch_cap < *n_batches_out) return HBP_ERR_CAPACITY;
    // emit in final order: batches as shuffled, their packs in sorted order
    int32_t n_item = 0, n_pack = 0;
    for (size_t b = 0; b < all_batches.size(); ++b) {
      const hbp_batch src = all_batches[b];
      batches[b] = hbp_batch{src.level, n_pack, src.n_packs, 0};
      for (int32_t k = 0; k < src.n_packs; ++k) {
        const Pack& pk = all_packs[src.first_pack + k];
        packs[n_pack++] = hbp_pack{src.level, n_item, (int32_t)pk.items.size(), pk.tokens, pk.attn};
        for (int32_t x : pk.items) pack_items[n_item++] = x;
      }
    }
  }
  if (metrics_or_null) {
    double dbr = 0.0, abr = 0.0;
    int64_t n_full = 0, pad = 0, capacity = 0, t_comm = 0, t_all = 0, devices = 0;
    for (const hbp_batch& b : all_batches) {
      std::vector<int64_t> tokens, attn;
      for (int32_t k = 0; k < b.n_packs; ++k) {
        tokens.push_back(all_packs[b.first_pack + k].tokens);
        attn.push_back(all_packs[b.first_pack + k].attn);
      }
      if (b.n_packs == packs_per_batch[b.level]) {
        dbr += ratio_to_max(tokens);
        abr += ratio_to_max(attn);
        ++n_full;
      }
      for (int64_t t : tokens) {
        pad += group_lens[b.level] - t;
        t_all += t;
        if (level_sp && level_sp[b.level] > 1) t_comm += t;
      }
      capacity += (int64_t)group_lens[b.level] * b.n_packs;
      devices += b.n_packs;
    }
    metrics_or_null->dbr = n_full ? dbr / (double)n_full : 0.0;
    metrics_or_null->abr = n_full ? abr / (double)n_full : 0.0;
    metrics_or_null->pr = capacity ? (double)pad / (double)capacity : 0.0;
    metrics_or_null->cr = t_all ? (double)t_comm / (double)t_all : 0.0;
    metrics_or_null->ave_t = devices ? (double)t_all / (double)devices : 0.0;
  }
  return HBP_OK;
}

// The planner allocates host memory: running out of it is reported, never thrown across the C boundary.
extern "C" hbp_status hbp_balance_packing(const int32_t* lengths, int32_t n_samples,
                                          const int32_t* group_lens, const int32_t* packs_per_batch,
                                          const int32_t* level_sp, int32_t n_levels,
                                          uint64_t shuffle_seed, int32_t* pack_items, int32_t item_cap,
                                          hbp_pack* packs, int32_t pack_cap, int32_t* n_packs_out,
                                          hbp_batch* batches, int32_t batch_cap, int32_t* n_batches_out,
                                          hbp_pack_metrics* metrics_or_null) {
  try {
    return hbp_balance_packing_impl(lengths, n_samples, group_lens, packs_per_batch, level_sp, n_levels, shuffle_seed,
                                    pack_items, item_cap, packs, pack_cap, n_packs_out, batches, batch_cap,
                                    n_batches_out, metrics_or_null);
  } catch (const std::bad_alloc&) {
    return HBP_ERR_NO_MEMORY;
  } catch (...) {
    return HBP_ERR_INVALID_ARG;
  }
}
