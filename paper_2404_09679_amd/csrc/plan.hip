// Host-side planning for heterogeneous dedicated devices (Section VI-B, Eq. 4): with gradient
// accumulation every device of type i computes C_i micro-batches of B_i samples one after the
// other before the synchronisation, and the plan minimises the longest of those sequences,
//   min max_i C_i * B_i / v_i   s.t.  sum_i n_i * C_i * B_i = B,
//   bmin_i <= B_i <= bmax_i,  cmin <= C_i <= cmax   (all integers).
// The accumulation counts are enumerated; for fixed counts the optimum over the batch sizes is
// found by bisection over the candidate values C_i * b / v_i, each tested with an exact
// bounded-coin reachability table over the sums  sum_i (n_i C_i) * B_i.
// A micro-batch is a shard of the global batch: accumulating a device's micro-batch
// gradients and then weighting the device by its share of B is the same sum as weighting
// every micro-batch by its own share, which is what antdt_aggregate computes.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <string>
#include <vector>

#include "common.h"

namespace {

struct Problem {
  int k;
  int64_t B;
  const int32_t* n;
  const double* v;
  const int64_t* bmin;
  const int64_t* bmax;
};

// cost(i, C, b) <= cost(j, Cj, bj) without division: C*b*v_j <= Cj*bj*v_i.
inline bool cost_le(long double cb_i, double v_i, long double cb_j, double v_j) {
  return cb_i * (long double)v_j <= cb_j * (long double)v_i;
}

// Is there B_i in [bmin_i, ub_i] with sum_i a_i * B_i = B?  On success the smallest feasible
// batch sizes (last type first) are written to out.
bool reachable(const Problem& p, const std::vector<int64_t>& a, const std::vector<int64_t>& ub,
               std::vector<int64_t>* out) {
  int64_t T = p.B;
  for (int i = 0; i < p.k; ++i) {
    if (ub[i] < p.bmin[i]) return false;
    T -= a[i] * p.bmin[i];
  }
  if (T < 0) return false;
  // layer[i][t]: t is a sum of the first i types' extra samples
  std::vector<std::vector<uint8_t>> layer(p.k + 1, std::vector<uint8_t>((size_t)T + 1, 0));
  std::vector<int64_t> used((size_t)T + 1);
  layer[0][0] = 1;
  for (int i = 0; i < p.k; ++i) {
    const int64_t cnt = ub[i] - p.bmin[i], w = a[i];
    for (int64_t t = 0; t <= T; ++t) {
      if (layer[i][t]) {
        layer[i + 1][t] = 1;
        used[t] = 0;
      } else if (t >= w && layer[i + 1][t - w] && used[t - w] < cnt) {
        layer[i + 1][t] = 1;
        used[t] = used[t - w] + 1;
      } else {
        used[t] = 0;
      }
    }
  }
  if (!layer[p.k][T]) return false;
  if (out) {
    out->assign(p.k, 0);
    int64_t t = T;
    for (int i = p.k - 1; i >= 0; --i) {
      int64_t x = 0;
      while (!(t - x * a[i] >= 0 && layer[i][t - x * a[i]])) ++x;  // exists: layer[i+1][t] holds
      (*out)[i] = p.bmin[i] + x;
      t -= x * a[i];
    }
  }
  return true;
}

}  // namespace

extern "C" {

int antdt_plan_accumulation(int64_t B, int32_t k, const int32_t* n, const double* v, const int64_t* bmin,
                            const int64_t* bmax, int32_t cmin, int32_t cmax, int64_t* B_out, int32_t* C_out,
                            double* z_out) {
  auto bad = [&](const char* what) {
    antdt::set_last_error(std::string("antdt_plan_accumulation: ") + what);
    return ANTDT_INVALID_ARG;
  };
  if (!n || !v || !bmin || !bmax || !B_out || !C_out) return bad("null argument");
  if (k < 1 || k > 8) return bad("number of device types must be 1..8");
  if (B < 1 || B > (1ll << 24)) return bad("B must be 1..2^24");
  if (cmin < 1 || cmax < cmin || cmax > 64) return bad("accumulation counts must satisfy 1 <= cmin <= cmax <= 64");
  double combos = 1;
  for (int i = 0; i < k; ++i) {
    if (n[i] < 1) return bad("device counts must be >= 1");
    if (!(v[i] > 0.0) || !std::isfinite(v[i])) return bad("speeds must be finite and > 0");
    if (bmin[i] < 1 || bmax[i] < bmin[i]) return bad("batch bounds must satisfy 1 <= bmin <= bmax");
    combos *= (double)(cmax - cmin + 1);
  }
  if (combos > 262144) return bad("too many combinations of accumulation counts");
  Problem p{k, B, n, v, bmin, bmax};
  bool have = false;
  long double best_cb = 0;  // the optimum as C*b of type best_i
  int best_i = 0;
  std::vector<int64_t> bestB;
  std::vector<int32_t> bestC, C(k, cmin);
  std::vector<int64_t> a(k), ub(k), sol;
  struct Cand { long double cb; int i; };
  std::vector<Cand> cand;
  for (;;) {
    for (int i = 0; i < k; ++i) a[i] = (int64_t)n[i] * C[i];
    // feasible at all?  (all upper bounds at bmax)
    for (int i = 0; i < k; ++i) ub[i] = bmax[i];
    int64_t lo_sum = 0, hi_sum = 0;
    for (int i = 0; i < k; ++i) {
      lo_sum += a[i] * bmin[i];
      hi_sum += a[i] * std::min<int64_t>(bmax[i], B);
    }
    if (lo_sum <= B && hi_sum >= B) {
      // candidate optimum values: C_i * b / v_i for every type and batch size, ascending
      cand.clear();
      for (int i = 0; i < k; ++i)
        for (int64_t b = bmin[i]; b <= std::min<int64_t>(bmax[i], B); ++b) cand.push_back({(long double)C[i] * b, i});
      std::sort(cand.begin(), cand.end(), [&](const Cand& x, const Cand& y) {
        return x.cb * (long double)v[y.i] < y.cb * (long double)v[x.i];
      });
      auto bounds_for = [&](const Cand& z) {
        for (int j = 0; j < k; ++j) {
          // largest b with C_j * b / v_j <= z
          int64_t b = (int64_t)floorl(z.cb * (long double)v[j] / ((long double)v[z.i] * C[j]));
          while (b + 1 <= bmax[j] && cost_le((long double)C[j] * (b + 1), v[j], z.cb, v[z.i])) ++b;
          while (b >= 0 && !cost_le((long double)C[j] * b, v[j], z.cb, v[z.i])) --b;
          ub[j] = std::min<int64_t>(b, bmax[j]);
        }
      };
      int64_t lo = 0, hi = (int64_t)cand.size() - 1;
      bounds_for(cand[hi]);
      if (reachable(p, a, ub, nullptr)) {
        while (lo < hi) {  // smallest candidate that is feasible (feasibility is monotone in z)
          const int64_t mid = (lo + hi) / 2;
          bounds_for(cand[mid]);
          if (reachable(p, a, ub, nullptr)) hi = mid; else lo = mid + 1;
        }
        const Cand& z = cand[lo];
        const bool better = !have || (z.cb * (long double)v[best_i] < best_cb * (long double)v[z.i]);
        if (better) {
          bounds_for(z);
          reachable(p, a, ub, &sol);
          have = true;
          best_cb = z.cb;
          best_i = z.i;
          bestB = sol;
          bestC = C;
        }
      }
    }
    int d = k - 1;  // next combination of accumulation counts, last type fastest
    while (d >= 0 && C[d] == cmax) C[d--] = cmin;
    if (d < 0) break;
    ++C[d];
  }
  if (!have) {
    antdt::set_last_error("antdt_plan_accumulation: no plan satisfies the constraints");
    return ANTDT_INFEASIBLE;
  }
  for (int i = 0; i < k; ++i) {
    B_out[i] = bestB[i];
    C_out[i] = bestC[i];
  }
  if (z_out) *z_out = (double)(best_cb / (long double)v[best_i]);
  return ANTDT_OK;
}

int antdt_expand_accumulation(int32_t k, const int32_t* n, const int64_t* Bi, const int32_t* Ci, int32_t cap,
                              int64_t* sizes_out, int32_t* device_out, int32_t* count_out) {
  if (!n || !Bi || !Ci || !sizes_out || !count_out || k < 1) {
    antdt::set_last_error("antdt_expand_accumulation: invalid argument");
    return ANTDT_INVALID_ARG;
  }
  int64_t total = 0;
  for (int i = 0; i < k; ++i) {
    if (n[i] < 0 || Ci[i] < 0 || Bi[i] < 0) {
      antdt::set_last_error("antdt_expand_accumulation: negative entry");
      return ANTDT_INVALID_ARG;
    }
    total += (int64_t)n[i] * Ci[i];
  }
  if (total > cap) {
    antdt::set_last_error("antdt_expand_accumulation: more micro-batches than the output arrays hold");
    return ANTDT_INVALID_ARG;
  }
  int32_t pos = 0, dev = 0;
  for (int i = 0; i < k; ++i)
    for (int d = 0; d < n[i]; ++d, ++dev)
      for (int c = 0; c < Ci[i]; ++c, ++pos) {
        sizes_out[pos] = Bi[i];
        if (device_out) device_out[pos] = dev;
      }
  *count_out = pos;
  return ANTDT_OK;
}

}  // extern "C"
