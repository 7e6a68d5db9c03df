// Balanced pipeline partitioning (Algorithm 1, Sec. III-C), host only.
//
// The network is seen as a queue of jobs, last layer first: for every layer a divisible job (its delta task,
// Eq. 4, which only the processor of the following layer may take over) followed by an atomic job (forward +
// weight gradient, which cannot move).  The jobs are packed into a row of bins of capacity T_p, one bin per
// processor, never returning to an earlier bin:
//   * a divisible job is poured into the open bin; what overflows opens the next bin (one cut per job: the
//     part that stayed is delta'', executed by the following layer's processor, the overflow is delta');
//   * an atomic job goes into the open bin if all of it fits, else it opens the next bin.
// T_p starts at (sum of all job times) / N_p; while the packing needs more than N_p bins, T_p grows by the
// factor alpha and the packing is redone.  Bins are numbered from the back of the network while packing and
// renumbered front to back for the caller.
//
// Readings of the printed algorithm: a bin opened for an atomic job starts empty; "fits" tolerates a relative
// 1e-9 so that exact fits (as in the paper's own example, to table rounding) survive floating point.
#include "../../include/lp.h"

#include <new>
#include <vector>

namespace {

constexpr double kFitTol = 1e-9;

struct Bins {
  double cap;
  std::vector<double> load;
  explicit Bins(double cap_) : cap(cap_), load(1, 0.0) {}
  int open_bin() const { return (int)load.size() - 1; }
  double room() const { return cap - load.back(); }
  void next() { load.push_back(0.0); }
  // returns the amount the bin that was open on entry took
  double pour(double amount) {
    const double free_now = room();
    if (amount <= free_now * (1.0 + kFitTol)) {
      load.back() += amount;
      return amount;
    }
    const double stays = free_now > 0.0 ? free_now : 0.0;
    load.back() += stays;
    next();
    load.back() += amount - stays;
    return stays;
  }
  void drop(double amount) {
    if (amount > room() * (1.0 + kFitTol) + kFitTol * cap) next();
    load.back() += amount;
  }
};

// where the two jobs of one layer ended up (bins counted from the back of the network)
struct LayerPlace {
  int delta_first_bin = 0;   // bin that was open when the delta task arrived
  int delta_last_bin = 0;    // bin that holds its overflow (same bin if it was not cut)
  double delta_first_share = 1.0;
  int fix_bin = 0;
};

int pack(const double* t_fix, const double* t_flex, int L, double cap, std::vector<LayerPlace>& place, std::vector<double>& load) {
  Bins bins(cap);
  for (int l = L - 1; l >= 0; --l) {
    LayerPlace& p = place[l];
    p.delta_first_bin = bins.open_bin();
    const double kept = bins.pour(t_flex[l]);
    p.delta_last_bin = bins.open_bin();
    p.delta_first_share = p.delta_last_bin == p.delta_first_bin ? 1.0 : (t_flex[l] > 0.0 ? kept / t_flex[l] : 0.0);
    bins.drop(t_fix[l]);
    p.fix_bin = bins.open_bin();
  }
  load.swap(bins.load);
  return (int)load.size();
}

}  // namespace

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
  try {
    std::vector<LayerPlace> place(L);
    std::vector<double> load;
    double target = total / n_proc;
    int used = pack(t_fix, t_flex, L, target, place, load);
    for (int relaxations = 0; used > n_proc; ++relaxations) {
      if (relaxations >= 100000) return LP_ERR_STATE;
      target *= alpha;
      used = pack(t_fix, t_flex, L, target, place, load);
    }
    auto stage_of = [used](int bin) { return used - 1 - bin; };
    for (int l = 0; l < L; ++l) {
      const LayerPlace& p = place[l];
      stage_fix[l] = stage_of(p.fix_bin);
      stage_delta_rest[l] = stage_of(p.delta_last_bin);
      // borrowed: the share that stayed in the bin of the following layer's immovable job, when this layer's own
      // immovable job sits in another bin
      const bool by_next = l + 1 < L && t_flex[l] > 0.0 && p.delta_first_bin == place[l + 1].fix_bin && p.fix_bin != place[l + 1].fix_bin;
      borrowed_frac[l] = by_next ? p.delta_first_share : 0.0;
    }
    for (int s = 0; s < n_proc; ++s) stage_time[s] = s < used ? load[used - 1 - s] : 0.0;
    if (t_p_out) *t_p_out = target;
    return LP_OK;
  } catch (const std::bad_alloc&) {
    return LP_ERR_STATE;
  } catch (...) {
    return LP_ERR_STATE;
  }
}
