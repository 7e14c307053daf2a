// Run-time choice of the re-computation configuration (App. B): host code only, no device work.
#include "dsk_internal.h"

namespace {

inline int point_layers(const dsk_frontier_point_t& p) { return p.hi - p.lo; }

// the cheaper of two points: fewer recomputed layers, then better quality, then the earlier one
inline bool cheaper(const dsk_frontier_point_t* f, int i, int best) {
  if (best < 0) return true;
  const int a = point_layers(f[i]), b = point_layers(f[best]);
  return a < b || (a == b && f[i].quality > f[best].quality);
}

inline bool richer(const dsk_frontier_point_t* f, int i, int best) {
  if (best < 0) return true;
  const int a = point_layers(f[i]), b = point_layers(f[best]);
  return a > b || (a == b && f[i].quality > f[best].quality);
}

}  // namespace

double dsk_estimate_prefill_ms(const dsk_latency_model_t* lat, int n_layers, int n_recomputed, int64_t n_tokens) {
  if (!lat) return 0.0;
  const double T = (double)n_tokens;
  return lat->c0 + n_recomputed * (lat->c_layer_token * T + lat->c_layer_token2 * T * T) +
         (n_layers - n_recomputed) * lat->c_reused_token * T;
}

int dsk_select_recompute(const dsk_frontier_point_t* frontier, int n_points, int n_layers, int64_t n_tokens,
                         const dsk_latency_model_t* lat, double slo_ms, double quality_target, int n_waiting,
                         int* chosen) {
  if (!frontier || n_points < 1 || n_layers < 1 || n_tokens < 0 || !lat || !chosen || n_waiting < 0) return DSK_EINVAL;
  for (int i = 0; i < n_points; ++i)
    if (!(0 <= frontier[i].lo && frontier[i].lo <= frontier[i].hi && frontier[i].hi <= n_layers)) return DSK_EINVAL;
  int cheapest = -1;
  for (int i = 0; i < n_points; ++i)
    if (cheaper(frontier, i, cheapest)) cheapest = i;
  int best = -1;
  if (n_waiting > 0) {
    // high load: the fewest recomputed layers that still reach the accuracy target
    for (int i = 0; i < n_points; ++i)
      if (frontier[i].quality >= quality_target && cheaper(frontier, i, best)) best = i;
  } else {
    // idle: the most recomputed layers whose estimated prefill delay meets the SLO
    for (int i = 0; i < n_points; ++i)
      if (dsk_estimate_prefill_ms(lat, n_layers, point_layers(frontier[i]), n_tokens) <= slo_ms && richer(frontier, i, best))
        best = i;
  }
  *chosen = best >= 0 ? best : cheapest;
  return DSK_OK;
}
