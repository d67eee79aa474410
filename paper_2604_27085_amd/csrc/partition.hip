// Automatic stage partitioning (paper Sec. 4.4): asymmetric forward / backward partitions of a layer sequence that
// minimise (M S + N (N - 1)) t_max under a per-stage memory limit.  Host code only.
#include <stddef.h>
#include <vector>

#include "../../include/rp.h"

namespace {

struct Split {
  std::vector<int> fwd, bwd;   // layers per forward stage (front to back); per backward stage (B_1 = the last layers first)
  double t_max = 0;
  bool ok = false;
};

// Greedy packing for one bound t: the fused first backward stage takes as many of the last layers as fit, the other
// backward stages follow towards the front, the forward stages cover what is left from the front.
Split pack(int L, const double* tf, const double* tb, const double* mf, const double* mb, double mem, double t) {
  Split s;
  int hi = L;   // backward stages cover [.., hi)
  while (hi > 0) {
    double st = 0, sm = 0;
    int n = 0;
    while (hi - n > 0 && st + tb[hi - n - 1] <= t && sm + mb[hi - n - 1] <= mem) { st += tb[hi - n - 1]; sm += mb[hi - n - 1]; ++n; }
    if (n == 0) return s;   // a single layer does not fit
    s.bwd.push_back(n);
    if (st > s.t_max) s.t_max = st;
    hi -= n;
  }
  const int lf = L - s.bwd[0];   // forward stages cover [0, lf)
  int lo = 0;
  while (lo < lf) {
    double st = 0, sm = 0;
    int n = 0;
    while (lo + n < lf && st + tf[lo + n] <= t && sm + mf[lo + n] <= mem) { st += tf[lo + n]; sm += mf[lo + n]; ++n; }
    if (n == 0) return s;
    s.fwd.push_back(n);
    if (st > s.t_max) s.t_max = st;
    lo += n;
  }
  s.ok = true;
  return s;
}

}  // namespace

extern "C" rp_status rp_partition_stages(int n_layers, const double* t_fwd, const double* t_bwd, const double* mem_fwd,
                                         const double* mem_bwd, double mem_limit, int n_gpus, int n_micro, int* fwd_layers,
                                         int* n_fwd, int* bwd_layers, int* n_bwd, double* t_max, double* cost) {
  if (n_layers <= 0 || !t_fwd || !t_bwd || !mem_fwd || !mem_bwd || n_gpus <= 0 || n_micro <= 0 || !fwd_layers || !n_fwd ||
      !bwd_layers || !n_bwd)
    return RP_EINVAL;
  for (int l = 0; l < n_layers; ++l)
    if (!(t_fwd[l] >= 0) || !(t_bwd[l] >= 0) || !(mem_fwd[l] >= 0) || !(mem_bwd[l] >= 0)) return RP_EINVAL;
  const int L = n_layers;
  const double bubble = (double)n_gpus * (n_gpus - 1);
  Split best;
  double best_cost = 0;
  auto consider = [&](double t) {
    const Split s = pack(L, t_fwd, t_bwd, mem_fwd, mem_bwd, mem_limit, t);
    if (!s.ok) return;
    const double S = (double)(s.fwd.size() + s.bwd.size());
    const double c = ((double)n_micro * S + bubble) * s.t_max;
    const bool better = !best.ok || c < best_cost ||
                        (c == best_cost && (s.fwd.size() + s.bwd.size() < best.fwd.size() + best.bwd.size()));
    if (better) { best = s; best_cost = c; }
  };
  // every contiguous run of forward times and of backward times is a candidate for the longest stage
  for (int which = 0; which < 2; ++which) {
    const double* tt = which ? t_bwd : t_fwd;
    for (int i = 0; i < L; ++i) {
      double sum = 0;
      for (int j = i; j < L; ++j) { sum += tt[j]; consider(sum); }
    }
  }
  if (!best.ok) return RP_EUNSUPPORTED;   // some layer exceeds the memory limit on its own
  *n_fwd = (int)best.fwd.size();
  *n_bwd = (int)best.bwd.size();
  for (size_t i = 0; i < best.fwd.size(); ++i) fwd_layers[i] = best.fwd[i];
  for (size_t i = 0; i < best.bwd.size(); ++i) bwd_layers[i] = best.bwd[i];
  if (t_max) *t_max = best.t_max;
  if (cost) *cost = best_cost;
  return RP_OK;
}
