// Host-side planning: layer-rate allocation (Sec. 4.1 Eq. 6-9) and per-layer token selection
// (Sec. 4.2: leading floor(r*T) tokens of each image; Sec. 4.1: rates non-increasing with depth).
#include <vector>

#include "vlc_internal.h"

using vlc::fail;

extern "C" int vlc_plan_layer_rates(int L, int G, const double* sens, int64_t budget_steps,
                                    int32_t* k_out) {
  if (!sens || !k_out) return fail(VLC_ERR_NULL, "vlc_plan_layer_rates: NULL pointer");
  if (L <= 0 || G <= 0 || G > VLC_RATE_GRID)
    return fail(VLC_ERR_SHAPE, "vlc_plan_layer_rates: L=%d G=%d out of range", L, G);
  if (budget_steps < 0) return fail(VLC_ERR_SHAPE, "vlc_plan_layer_rates: negative budget");
  const int64_t stride = (int64_t)G + 1;
  for (int i = 0; i < L; ++i) k_out[i] = 0;
  for (int64_t used = 0; used < budget_steps; ++used) {
    int pick = -1;
    double pick_drop = 0.0;
    for (int i = 0; i < L; ++i) {
      const int32_t ki = k_out[i];
      if (ki >= G) continue;                            // grid ceiling (Eq. 9)
      if (i > 0 && ki + 1 > k_out[i - 1]) continue;     // r_i <= r_{i-1} (Eq. 8)
      // one IEEE subtraction of two stored doubles: identical on every conforming host
      volatile double drop = sens[i * stride + ki] - sens[i * stride + ki + 1];
      if (drop > pick_drop) {                           // strict: ties stay with the lower index
        pick = i;
        pick_drop = drop;
      }
    }
    if (pick < 0) break;                                // nothing left that lowers the objective
    k_out[pick] += 1;
  }
  return VLC_OK;
}

extern "C" int vlc_plan_layer_rates_blocks(int L, int G, const double* sens, int64_t budget_steps,
                                           int32_t* k_out) {
  if (!sens || !k_out) return fail(VLC_ERR_NULL, "vlc_plan_layer_rates_blocks: NULL pointer");
  if (L <= 0 || G <= 0 || G > VLC_RATE_GRID)
    return fail(VLC_ERR_SHAPE, "vlc_plan_layer_rates_blocks: L=%d G=%d out of range", L, G);
  if (budget_steps < 0) return fail(VLC_ERR_SHAPE, "vlc_plan_layer_rates_blocks: negative budget");
  const int64_t stride = (int64_t)G + 1;
  for (int i = 0; i < L; ++i) k_out[i] = 0;
  int64_t used = 0;
  while (used < budget_steps) {
    int best_j = -1, best_a = 0, best_cost = 1;
    double best_gain = 0.0;
    for (int j = 0; j < L; ++j) {
      if (k_out[j] >= G) continue;                          // grid ceiling (Eq. 9)
      int a = j;                                            // layers a..j-1 sit at j's level: they rise with it (Eq. 8)
      while (a > 0 && k_out[a - 1] == k_out[j]) --a;
      const int cost = j - a + 1;
      if (used + cost > budget_steps) continue;             // Eq. 7
      volatile double gain = 0.0;                           // every operation a plain IEEE one, in layer order
      for (int i = a; i <= j; ++i) {
        volatile double drop = sens[i * stride + k_out[i]] - sens[i * stride + k_out[i] + 1];
        gain = gain + drop;
      }
      if (!(gain > 0.0)) continue;
      volatile double lhs = gain * (double)best_cost, rhs = best_gain * (double)cost;
      if (best_j < 0 || lhs > rhs) {                        // more gain per step; equal: the smaller j stays
        best_j = j;
        best_a = a;
        best_gain = gain;
        best_cost = cost;
      }
    }
    if (best_j < 0) break;
    for (int i = best_a; i <= best_j; ++i) k_out[i] += 1;
    used += best_cost;
  }
  return VLC_OK;
}

namespace {

int check_segments(int n_seg, const vlc_segment* seg, const char* who) {
  if (n_seg <= 0) return fail(VLC_ERR_SHAPE, "%s: n_seg=%d", who, n_seg);
  for (int s = 0; s < n_seg; ++s) {
    const vlc_segment& g = seg[s];
    if (g.length < 0 || g.start < 0 || g.kv_start < 0 || g.start < g.kv_start)
      return fail(VLC_ERR_INDEX, "%s: segment %d has a negative or inconsistent field", who, s);
    if (g.is_image && g.cache_row < 0)
      return fail(VLC_ERR_INDEX, "%s: segment %d has a negative cache_row", who, s);
    if (s > 0) {
      const vlc_segment& p = seg[s - 1];
      if (g.start < p.start + p.length)
        return fail(VLC_ERR_INDEX, "%s: segments %d and %d overlap or are out of order", who, s - 1, s);
      if (g.kv_start < p.kv_start)
        return fail(VLC_ERR_INDEX, "%s: requests are not in ascending order at segment %d", who, s);
    }
  }
  return VLC_OK;
}

// leading tokens of a T-token image recomputed at layer l
inline int64_t leading(const int32_t* k, const int32_t* over, int l, int64_t T) {
  if (over) return over[l] < T ? (over[l] < 0 ? 0 : over[l]) : T;
  return ((int64_t)k[l] * T) / VLC_RATE_GRID;           // floor(r*T), r = k/500 (Sec. 4.2)
}

int check_rates(int L, const int32_t* k, const int32_t* over, const char* who) {
  if (!k && !over) return fail(VLC_ERR_NULL, "%s: k and count_override are both NULL", who);
  for (int l = 0; l < L; ++l) {
    if (over) {
      if (over[l] < 0) return fail(VLC_ERR_SHAPE, "%s: count_override[%d] < 0", who, l);
      if (l > 0 && over[l] > over[l - 1])
        return fail(VLC_ERR_INFEASIBLE, "%s: layer %d recomputes more than layer %d", who, l, l - 1);
    } else {
      if (k[l] < 0 || k[l] > VLC_RATE_GRID)
        return fail(VLC_ERR_SHAPE, "%s: k[%d]=%d outside 0..%d", who, l, k[l], VLC_RATE_GRID);
      if (l > 0 && k[l] > k[l - 1])
        return fail(VLC_ERR_INFEASIBLE, "%s: rate of layer %d exceeds layer %d (must not increase)",
                    who, l, l - 1);
    }
  }
  return VLC_OK;
}

}  // namespace

extern "C" int vlc_plan_token_indices(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                                      const int32_t* count_override, int64_t cap, int32_t* n_rows,
                                      int32_t* slot, int32_t* map, int32_t* pos, int32_t* kv_start,
                                      int32_t* kv_len) {
  const char* who = "vlc_plan_token_indices";
  if (!seg || !n_rows) return fail(VLC_ERR_NULL, "%s: NULL pointer", who);
  if (L <= 0 || cap < 0) return fail(VLC_ERR_SHAPE, "%s: L=%d cap=%lld", who, L, (long long)cap);
  int rc = check_segments(n_seg, seg, who);
  if (rc) return rc;
  rc = check_rates(L, k, count_override, who);
  if (rc) return rc;

  // Rows kept by the previous layer, as (segment, offset) runs: because only a *leading* part of
  // each image is kept and the counts never grow, the position of a token in the previous layer's
  // row list is (rows before its segment in that list) + (its offset inside the segment).
  std::vector<int64_t> prev_before(n_seg, 0);   // rows of the previous layer before segment s
  std::vector<int64_t> cur_before(n_seg, 0);
  for (int l = 0; l < L; ++l) {
    int64_t n = 0;
    for (int s = 0; s < n_seg; ++s) {
      const vlc_segment& g = seg[s];
      const int64_t take = g.is_image ? leading(k, count_override, l, g.length) : g.length;
      cur_before[s] = n;
      if (n + take > cap) return fail(VLC_ERR_SHAPE, "%s: cap=%lld too small at layer %d", who,
                                      (long long)cap, l);
      for (int64_t t = 0; t < take; ++t) {
        const int64_t o = (int64_t)l * cap + n + t;
        const int32_t sl = (int32_t)(g.start + t);
        if (slot) slot[o] = sl;
        if (map) map[o] = l == 0 ? sl : (int32_t)(prev_before[s] + t);
        if (pos) pos[o] = (int32_t)(g.pos + t);
        if (kv_start) kv_start[o] = g.kv_start;
        if (kv_len) kv_len[o] = sl - g.kv_start + 1;
      }
      n += take;
    }
    n_rows[l] = (int32_t)n;
    prev_before.swap(cur_before);
  }
  return VLC_OK;
}

extern "C" int vlc_plan_next_rows(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                                  const int32_t* count_override, int64_t cap, int32_t* next_row) {
  const char* who = "vlc_plan_next_rows";
  if (!seg || !next_row) return fail(VLC_ERR_NULL, "%s: NULL pointer", who);
  if (L <= 0 || cap < 0) return fail(VLC_ERR_SHAPE, "%s: L=%d cap=%lld", who, L, (long long)cap);
  int rc = check_segments(n_seg, seg, who);
  if (rc) return rc;
  rc = check_rates(L, k, count_override, who);
  if (rc) return rc;
  // A layer keeps the leading take(l) tokens of a segment, the layer below the leading take(l+1) <= take(l) of
  // them: row (rows of layer l before the segment) + t goes to (rows of layer l+1 before it) + t if t < take(l+1).
  for (int l = 0; l < L; ++l) {
    int64_t n = 0, n_below = 0;
    for (int s = 0; s < n_seg; ++s) {
      const vlc_segment& g = seg[s];
      const int64_t take = g.is_image ? leading(k, count_override, l, g.length) : g.length;
      const int64_t below = l + 1 >= L ? 0 : (g.is_image ? leading(k, count_override, l + 1, g.length) : g.length);
      if (n + take > cap) return fail(VLC_ERR_SHAPE, "%s: cap=%lld too small at layer %d", who, (long long)cap, l);
      for (int64_t t = 0; t < take; ++t)
        next_row[(int64_t)l * cap + n + t] = t < below ? (int32_t)(n_below + t) : -1;
      n += take;
      n_below += below;
    }
  }
  return VLC_OK;
}

extern "C" int vlc_plan_budget_steps(int mean_rate_bp, int L, int64_t* steps) {
  if (!steps) return fail(VLC_ERR_NULL, "vlc_plan_budget_steps: steps is NULL");
  if (mean_rate_bp < 0 || mean_rate_bp > 10000 || L <= 0)
    return fail(VLC_ERR_SHAPE, "vlc_plan_budget_steps: mean_rate_bp=%d (0..10000) L=%d", mean_rate_bp, L);
  // a mean rate of bp / 10000 over L layers is a rate sum of bp * L / 10000 (Eq. 7), i.e. bp * L / 20 grid steps
  *steps = ((int64_t)mean_rate_bp * L) / (10000 / VLC_RATE_GRID);
  return VLC_OK;
}

extern "C" int vlc_plan_reuse_rows(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                                   const int32_t* count_override, int64_t cap, int32_t* n_reuse,
                                   int32_t* src_row, int32_t* dst_slot, int32_t* delta) {
  const char* who = "vlc_plan_reuse_rows";
  if (!seg || !n_reuse) return fail(VLC_ERR_NULL, "%s: NULL pointer", who);
  if (L <= 0 || cap < 0) return fail(VLC_ERR_SHAPE, "%s: L=%d cap=%lld", who, L, (long long)cap);
  int rc = check_segments(n_seg, seg, who);
  if (rc) return rc;
  rc = check_rates(L, k, count_override, who);
  if (rc) return rc;
  for (int l = 0; l < L; ++l) {
    int64_t n = 0;
    for (int s = 0; s < n_seg; ++s) {
      const vlc_segment& g = seg[s];
      if (!g.is_image) continue;
      const int64_t first = leading(k, count_override, l, g.length);
      if (n + (g.length - first) > cap)
        return fail(VLC_ERR_SHAPE, "%s: cap=%lld too small at layer %d", who, (long long)cap, l);
      for (int64_t t = first; t < g.length; ++t, ++n) {
        const int64_t o = (int64_t)l * cap + n;
        if (src_row) src_row[o] = (int32_t)(g.cache_row + t);
        if (dst_slot) dst_slot[o] = (int32_t)(g.start + t);
        if (delta) delta[o] = g.pos - g.old_pos;          // same for every token of the run
      }
    }
    n_reuse[l] = (int32_t)n;
  }
  return VLC_OK;
}
