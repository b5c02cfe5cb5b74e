// Driver for the host-only entry points (pack plan, Balance Packing, auto-selection) built with
// AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py: seeded random and
// edge-case inputs, exact-size output buffers (so an overrun by one element is caught), size queries,
// error paths.  Prints "ok" and returns 0 when every call returned the expected status.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "hbp.h"

static uint64_t rng_state = 0x1234567;
static uint32_t rnd() {
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(rng_state >> 33);
}
#define CHECK(cond)                                                   \
  do {                                                                \
    if (!(cond)) {                                                    \
      std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                       \
    }                                                                 \
  } while (0)

static double prof_memory(void*, int32_t l, int32_t sp, int32_t c) { return 30.0 - 0.002 * l / sp * (32 - c) / 32.0; }
static double prof_time(void*, int32_t l, int32_t sp, int32_t c) { return 1.0 + l * 1e-5 + 0.05 * sp + 0.01 * c + 1000.0 / l; }
static double prof_oom(void*, int32_t, int32_t, int32_t) { return -1.0; }

int main() {
  // ---- hbp_pack_plan
  for (int round = 0; round < 200; ++round) {
    const int n = (int)(rnd() % 40);
    std::vector<int32_t> lens(n);
    for (auto& v : lens) v = 1 + (int32_t)(rnd() % 3000);
    const int32_t pack_len = 1 + (int32_t)(rnd() % 20000), rows = (rnd() & 1) ? 128 : 64, kind = rnd() & 1;
    int32_t ns = 0, nc = 0, nt = 0;
    int64_t pc = 0;
    CHECK(hbp_pack_plan(lens.data(), n, pack_len, rows, kind, nullptr, 0, &ns, &nc, nullptr, nullptr, 0, &nt, &pc) == HBP_OK);
    std::vector<int32_t> cu(ns + 1);
    std::vector<hbp_tile> tiles(nt);
    std::vector<int64_t> cost(nt);
    int32_t ns2 = 0, nc2 = 0, nt2 = 0;
    CHECK(hbp_pack_plan(lens.data(), n, pack_len, rows, kind, cu.data(), ns + 1, &ns2, &nc2, tiles.data(), cost.data(), nt,
                        &nt2, &pc) == HBP_OK);
    CHECK(ns2 == ns && nt2 == nt && nc2 == nc && cu[0] == 0 && cu[ns] <= pack_len);
    if (nt > 1) {  // one element short must be refused, not overrun (a NULL list is a size query)
      std::vector<hbp_tile> small(nt - 1);
      std::vector<int64_t> small_cost(nt - 1);
      CHECK(hbp_pack_plan(lens.data(), n, pack_len, rows, kind, cu.data(), ns + 1, &ns2, &nc2, small.data(),
                          small_cost.data(), nt - 1, &nt2, &pc) != HBP_OK);
    }
  }
  {
    int32_t bad[3] = {5, 0, 7}, ns, nc, nt;
    int64_t pc;
    CHECK(hbp_pack_plan(bad, 3, 100, 64, 0, nullptr, 0, &ns, &nc, nullptr, nullptr, 0, &nt, &pc) != HBP_OK);
    CHECK(hbp_pack_plan(nullptr, 0, 100, 64, 0, nullptr, 0, &ns, &nc, nullptr, nullptr, 0, &nt, &pc) == HBP_OK);
  }

  // ---- hbp_balance_packing
  for (int round = 0; round < 60; ++round) {
    const int n = (int)(rnd() % 3000);
    const int levels = 1 + (int)(rnd() % 4);
    std::vector<int32_t> groups(levels), per_batch(levels), sp(levels);
    int32_t g = 0;
    for (int i = 0; i < levels; ++i) {
      g += 256 + (int32_t)(rnd() % 4096);
      groups[i] = g;
      per_batch[i] = 1 + (int32_t)(rnd() % 8);
      sp[i] = 1 << (rnd() % 4);
    }
    std::vector<int32_t> lens(n);
    for (auto& v : lens) v = 1 + (int32_t)(rnd() % g);
    int32_t np = 0, nb = 0;
    hbp_pack_metrics m;
    CHECK(hbp_balance_packing(lens.data(), n, groups.data(), per_batch.data(), sp.data(), levels, rnd(), nullptr, 0,
                              nullptr, 0, &np, nullptr, 0, &nb, &m) == HBP_OK);
    std::vector<int32_t> items(n);
    std::vector<hbp_pack> packs(np);
    std::vector<hbp_batch> batches(nb);
    int32_t np2 = 0, nb2 = 0;
    CHECK(hbp_balance_packing(lens.data(), n, groups.data(), per_batch.data(), (round & 1) ? sp.data() : nullptr, levels,
                              7, items.data(), n, packs.data(), np, &np2, batches.data(), nb, &nb2, nullptr) == HBP_OK);
    CHECK(np2 == np && nb2 == nb);
    std::vector<char> seen(n, 0);
    for (int32_t x : items) {
      CHECK(x >= 0 && x < n && !seen[x]);
      seen[x] = 1;
    }
    if (np > 1) {
      std::vector<hbp_pack> small(np - 1);
      CHECK(hbp_balance_packing(lens.data(), n, groups.data(), per_batch.data(), nullptr, levels, 7, items.data(), n,
                                small.data(), np - 1, &np2, batches.data(), nb, &nb2, nullptr) != HBP_OK);
    }
    if (n > 0) {
      lens[rnd() % n] = g + 1;  // longer than the largest group
      CHECK(hbp_balance_packing(lens.data(), n, groups.data(), per_batch.data(), nullptr, levels, 7, nullptr, 0, nullptr,
                                0, &np2, nullptr, 0, &nb2, nullptr) != HBP_OK);
    }
  }

  // ---- hbp_auto_select
  {
    const int32_t lengths[5] = {8192, 16384, 32768, 65536, 131072}, sps[5] = {1, 2, 4, 8, 16};
    hbp_profile pr = {prof_memory, prof_time, nullptr};
    hbp_strategy per[5];
    hbp_group groups[4];
    int32_t ng = 0, j = -1;
    for (int nl = 1; nl <= 5; ++nl)
      for (int nsp = 1; nsp <= 5; ++nsp) {
        CHECK(hbp_auto_select(lengths, nl, sps, nsp, 20, 32, &pr, per, groups, &ng, &j) == HBP_OK);
        CHECK(ng >= 1 && ng <= 4 && j >= 0 && j < nl && groups[ng - 1].l == lengths[nl - 1]);
        for (int i = 1; i < ng; ++i) CHECK(groups[i].l > groups[i - 1].l);
        CHECK(hbp_auto_select(lengths, nl, sps, nsp, 20, 32, &pr, nullptr, groups, &ng, nullptr) == HBP_OK);
      }
    hbp_profile oom = {prof_oom, prof_time, nullptr};
    CHECK(hbp_auto_select(lengths, 5, sps, 5, 20, 32, &oom, per, groups, &ng, &j) == HBP_ERR_UNSUPPORTED);
    CHECK(hbp_auto_select(lengths, 5, sps, 5, 32, 32, &pr, per, groups, &ng, &j) == HBP_ERR_INVALID_ARG);
    CHECK(hbp_auto_select(lengths, 0, sps, 5, 20, 32, &pr, per, groups, &ng, &j) == HBP_ERR_INVALID_ARG);
    CHECK(hbp_auto_select(nullptr, 5, sps, 5, 20, 32, &pr, per, groups, &ng, &j) == HBP_ERR_INVALID_ARG);
  }
  std::puts("ok");
  return 0;
}
