// Hierarchical Groups Auto-Selection (Section 4.1, Algorithm 1; appendix "Implementation Details of
// Hierarchical Groups Auto-Selection": FindBestSpCkpt, GreedyProfileCkpt).  Host only; profiling
// comes from the caller's callbacks.
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>

#include "hbp.h"

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

// layers to checkpoint for (l, sp): zero crossing of the remaining memory, linear in the layer count
// between the two profiled points; -1 = does not fit
int32_t greedy_profile_ckpt(const hbp_profile& pr, int32_t l, int32_t sp, int32_t c_min, int32_t c_max) {
  const double m1 = pr.memory(pr.ctx, l, sp, c_min);
  const double m2 = pr.memory(pr.ctx, l, sp, c_max);
  if (!(m2 >= 0.0)) return -1;
  const double m_ave = (m2 - m1) / (double)(c_max - c_min);
  if (m_ave > 0.0) {
    const double c_o = std::ceil((double)c_max - m2 / m_ave);
    return c_o > 0.0 ? (int32_t)c_o : 0;
  }
  return m2 - m_ave * (double)c_max >= 0.0 ? 0 : -1;
}

hbp_strategy find_best_sp_ckpt(const hbp_profile& pr, int32_t l, const int32_t* sp_set, int32_t n_sp,
                               int32_t c_min, int32_t c_max) {
  hbp_strategy best = {l, 0, 0, 0, kInf};
  for (int32_t i = 0; i < n_sp; ++i) {
    const int32_t ckpt = greedy_profile_ckpt(pr, l, sp_set[i], c_min, c_max);
    if (ckpt < 0) continue;
    const double t = pr.time(pr.ctx, l, sp_set[i], ckpt);
    if (!(t >= 0.0) || !(t < kInf)) continue;
    if (!best.feasible || t < best.time) best = {l, sp_set[i], ckpt, 1, t};
  }
  return best;
}

}  // namespace

static hbp_status hbp_auto_select_impl(const int32_t* lengths, int32_t n_lengths, const int32_t* sp_set,
                                      int32_t n_sp, int32_t c_min, int32_t c_max, const hbp_profile* profile,
                                      hbp_strategy* per_length_or_null, hbp_group* groups,
                                      int32_t* n_groups_out, int32_t* best_index_out_or_null) {
  if (!lengths || !sp_set || !profile || !profile->memory || !profile->time || !groups || !n_groups_out)
    return HBP_ERR_INVALID_ARG;
  if (n_lengths < 1 || n_sp < 1 || c_min < 0 || c_min >= c_max) return HBP_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_lengths; ++i)
    if (lengths[i] <= 0 || (i > 0 && lengths[i] <= lengths[i - 1])) return HBP_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_sp; ++i)
    if (sp_set[i] <= 0) return HBP_ERR_INVALID_ARG;

  // Stage 1
  hbp_strategy best = {0, 0, 0, 0, kInf}, last = best;
  int32_t j = -1;
  for (int32_t i = 0; i < n_lengths; ++i) {
    const hbp_strategy s = find_best_sp_ckpt(*profile, lengths[i], sp_set, n_sp, c_min, c_max);
    if (per_length_or_null) per_length_or_null[i] = s;
    if (s.feasible && (j < 0 || s.time < best.time)) {
      best = s;
      j = i;
    }
    last = s;
  }
  if (!last.feasible) return HBP_ERR_UNSUPPORTED;

  // Stage 2
  const int32_t l_1 = best.l / best.sp, l_2 = last.l / last.sp;
  hbp_group cand[4];
  int32_t n = 0;
  cand[n++] = {l_1, 1, best.ckpt, 0};
  cand[n++] = {best.l, best.sp, best.ckpt, 0};
  if (l_2 > best.l) cand[n++] = {l_2, 1, last.ckpt, 0};
  cand[n++] = {last.l, last.sp, last.ckpt, 0};
  int32_t m = 0;
  for (int32_t i = 0; i < n; ++i) {  // a repeated length keeps the later entry: the length's own strategy
    if (m > 0 && groups[m - 1].l == cand[i].l) groups[m - 1] = cand[i];
    else groups[m++] = cand[i];
  }
  *n_groups_out = m;
  if (best_index_out_or_null) *best_index_out_or_null = j;
  return HBP_OK;
}

// The planner allocates host memory: running out of it is reported, never thrown across the C boundary.
extern "C" hbp_status hbp_auto_select(const int32_t* lengths, int32_t n_lengths, const int32_t* sp_set,
                                      int32_t n_sp, int32_t c_min, int32_t c_max, const hbp_profile* profile,
                                      hbp_strategy* per_length_or_null, hbp_group* groups,
                                      int32_t* n_groups_out, int32_t* best_index_out_or_null) {
  try {
    return hbp_auto_select_impl(lengths, n_lengths, sp_set, n_sp, c_min, c_max, profile, per_length_or_null, groups,
                                n_groups_out, best_index_out_or_null);
  } catch (const std::bad_alloc&) {
    return HBP_ERR_NO_MEMORY;
  } catch (...) {
    return HBP_ERR_INVALID_ARG;
  }
}
