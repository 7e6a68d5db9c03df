// Balanced pipeline partitioning (Algorithm 1, Sec. III-C), host only.
//
// Layers are walked from the last to the first while processors are filled up to the target load
// T_p = (sum of all task times) / N_p.  A layer contributes a movable delta task (only the processor
// of the following layer may take it over) and an immovable part (forward + weight gradient).  The
// delta task is offered first to the processor that is currently being filled, which is the one that
// holds the following layer; what does not fit (delta') opens the next processor.  The immovable part
// follows: into the current processor if it fits, else into a fresh one.  When the walk needs more
// than N_p processors, T_p grows by the factor alpha and the walk starts over.
//
// Readings of the printed algorithm: a processor opened for an immovable part starts empty; stages are
// renumbered front to back at the end; "fits" tolerates a relative 1e-9 so that exact fits (as in the
// paper's own example, to table rounding) survive floating point.
#include "../../include/lp.h"

#include <vector>

extern "C" int lp_partition(const double* t_fix, const double* t_flex, int L, int n_proc, double alpha, int* stage_fix,
                            int* stage_delta_rest, double* borrowed_frac, double* stage_time, double* t_p_out) {
  if (!t_fix || !t_flex || !stage_fix || !stage_delta_rest || !borrowed_frac || !stage_time) return LP_ERR_NULL;
  if (L < 1 || n_proc < 1 || !(alpha > 1.0)) return LP_ERR_SHAPE;
  double total = 0.0;
  for (int l = 0; l < L; ++l) {
    if (!(t_fix[l] >= 0.0) || !(t_flex[l] >= 0.0)) return LP_ERR_SHAPE;
    total += t_fix[l];
  }
  for (int l = 0; l < L; ++l) total += t_flex[l];
  const double slack = 1e-9;
  double target = total / n_proc;
  std::vector<int> fix_on(L), first_on(L), rest_on(L);
  std::vector<double> first_part(L);
  std::vector<double> load;
  for (int round = 0; round < 100000; ++round) {
    load.assign(1, 0.0);
    int cur = 0;
    double room = target;
    for (int l = L - 1; l >= 0; --l) {
      const double d = t_flex[l];
      first_on[l] = cur;
      if (d <= room * (1.0 + slack)) {
        load[cur] += d;
        room -= d;
        first_part[l] = 1.0;
        rest_on[l] = cur;
      } else {
        const double stays = room > 0.0 ? room : 0.0;   // delta''
        const double moves = d - stays;                 // delta'
        load[cur] += stays;
        first_part[l] = stays / d;
        load.push_back(moves);
        ++cur;
        room = target - moves;
        rest_on[l] = cur;
      }
      if (t_fix[l] > room * (1.0 + slack) + slack * target) {
        load.push_back(0.0);
        ++cur;
        room = target;
      }
      load[cur] += t_fix[l];
      room -= t_fix[l];
      fix_on[l] = cur;
    }
    const int used = cur + 1;
    if (used > n_proc) {
      target *= alpha;
      continue;
    }
    for (int l = 0; l < L; ++l) {
      stage_fix[l] = used - 1 - fix_on[l];
      stage_delta_rest[l] = used - 1 - rest_on[l];
      const bool borrowed = l < L - 1 && first_on[l] == fix_on[l + 1] && fix_on[l + 1] != fix_on[l] && t_flex[l] > 0.0;
      borrowed_frac[l] = borrowed ? first_part[l] : 0.0;
    }
    for (int s = 0; s < n_proc; ++s) stage_time[s] = s < used ? load[used - 1 - s] : 0.0;
    if (t_p_out) *t_p_out = target;
    return LP_OK;
  }
  return LP_ERR_STATE;
}
