// Host-side parts of the framework around the iteration (no GPU work):
//  * the shard queue with states of Section V-C (V-C.1 shards, V-C.3 states and re-queue): N samples cut into K = ceil(N / (B*M)) shards
//    (start, length), TODO -> DOING (fetched by a worker) -> DONE (its gradients were pushed);
//    the DOING shards of a lost worker go back to TODO at the END of the queue;
//  * an iteration-level model of bulk-synchronous training under injected stragglers: one
//    iteration takes max_i T_i + T_server with T_i = t0_i + B_i / v_i + delay_i and sum B_i = B
//    (Eq. 1, server and communication terms lumped together), delays injected as in
//    Section VII-A.2, policies BSP / ADJUST_BS (Eq. 3) / BACKUP_WORKERS / ADJUST_BS +
//    KILL_RESTART (Section VI-A).  See antdt.h for the exact rules.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <deque>
#include <string>
#include <vector>

#include "common.h"

struct antdt_dds {
  std::vector<int64_t> start, len;
  std::vector<int32_t> state, owner;
  std::deque<int64_t> queue;
};

namespace {

int bad(const char* fn, const char* what) {
  antdt::set_last_error(std::string(fn) + ": " + what);
  return ANTDT_INVALID_ARG;
}

inline uint32_t fmix32(uint32_t x) {  // MurmurHash3's 32-bit finaliser
  x ^= x >> 16;
  x *= 0x85EBCA6Bu;
  x ^= x >> 13;
  x *= 0xC2B2AE35u;
  x ^= x >> 16;
  return x;
}

inline bool disturbed(uint32_t seed, int64_t window, int worker, double prob) {
  const uint32_t u = fmix32(seed ^ fmix32((uint32_t)((uint64_t)window * 0x9E3779B9ull + (uint64_t)worker + 1ull)));
  return (double)u / 4294967296.0 < prob;
}

// Eq. 3 in double precision: floor(B v_i / sum v) - 1 each, the rest one sample at a time to
// the worker whose load after the addition is smallest (ties: lowest index).
void split_by_speed(int64_t B, const std::vector<double>& v, std::vector<int64_t>& out) {
  double tot = 0.0;
  for (double x : v) tot += x;
  out.assign(v.size(), 0);
  int64_t given = 0;
  for (size_t i = 0; i < v.size(); ++i) {
    int64_t b = (int64_t)floor(((double)B * v[i]) / tot) - 1;
    if (b < 0) b = 0;
    out[i] = b;
    given += b;
  }
  for (; given < B; ++given) {
    size_t best = 0;
    for (size_t k = 1; k < v.size(); ++k)
      if ((double)(out[k] + 1) * v[best] < (double)(out[best] + 1) * v[k]) best = k;
    ++out[best];
  }
}

struct Rec {
  double t_end;
  int64_t b;
  double T;
};

}  // namespace

extern "C" {

int antdt_dds_create(int64_t N, int64_t B, int32_t M, antdt_dds** out) {
  if (!out) return bad("antdt_dds_create", "null argument");
  if (N < 0 || B < 1 || M < 1) return bad("antdt_dds_create", "N >= 0, B >= 1 and M >= 1 required");
  const int64_t per = B * (int64_t)M;
  const int64_t K = (N + per - 1) / per;
  if (K > (1ll << 28)) return bad("antdt_dds_create", "too many shards");
  antdt_dds* d = new antdt_dds();
  d->start.resize(K);
  d->len.resize(K);
  d->state.assign(K, ANTDT_SHARD_TODO);
  d->owner.assign(K, -1);
  for (int64_t k = 0; k < K; ++k) {
    d->start[k] = k * per;
    d->len[k] = std::min(per, N - k * per);
    d->queue.push_back(k);
  }
  *out = d;
  return ANTDT_OK;
}

int antdt_dds_destroy(antdt_dds* d) {
  delete d;
  return ANTDT_OK;
}

int antdt_dds_num_shards(const antdt_dds* d, int64_t* K) {
  if (!d || !K) return bad("antdt_dds_num_shards", "null argument");
  *K = (int64_t)d->start.size();
  return ANTDT_OK;
}

int antdt_dds_fetch(antdt_dds* d, int32_t worker, int64_t* shard, int64_t* start, int64_t* len) {
  if (!d || !shard || !start || !len) return bad("antdt_dds_fetch", "null argument");
  if (worker < 0) return bad("antdt_dds_fetch", "worker index must be >= 0");
  if (d->queue.empty()) {
    antdt::set_last_error("antdt_dds_fetch: no shard is waiting");
    return ANTDT_EMPTY;
  }
  const int64_t k = d->queue.front();
  d->queue.pop_front();
  d->state[k] = ANTDT_SHARD_DOING;
  d->owner[k] = worker;
  *shard = k;
  *start = d->start[k];
  *len = d->len[k];
  return ANTDT_OK;
}

int antdt_dds_report_done(antdt_dds* d, int64_t shard, int32_t worker) {
  if (!d) return bad("antdt_dds_report_done", "null argument");
  if (shard < 0 || shard >= (int64_t)d->start.size()) return bad("antdt_dds_report_done", "shard index out of range");
  if (d->state[shard] != ANTDT_SHARD_DOING || d->owner[shard] != worker) {
    antdt::set_last_error("antdt_dds_report_done: the shard is not being worked on by this worker");
    return ANTDT_BAD_STATE;
  }
  d->state[shard] = ANTDT_SHARD_DONE;
  d->owner[shard] = -1;
  return ANTDT_OK;
}

int antdt_dds_release_worker(antdt_dds* d, int32_t worker, int64_t* requeued) {
  if (!d) return bad("antdt_dds_release_worker", "null argument");
  int64_t n = 0;
  for (int64_t k = 0; k < (int64_t)d->start.size(); ++k)
    if (d->state[k] == ANTDT_SHARD_DOING && d->owner[k] == worker) {
      d->state[k] = ANTDT_SHARD_TODO;
      d->owner[k] = -1;
      d->queue.push_back(k);
      ++n;
    }
  if (requeued) *requeued = n;
  return ANTDT_OK;
}

int antdt_dds_shard(const antdt_dds* d, int64_t shard, int64_t* start, int64_t* len, int32_t* state, int32_t* owner) {
  if (!d) return bad("antdt_dds_shard", "null argument");
  if (shard < 0 || shard >= (int64_t)d->start.size()) return bad("antdt_dds_shard", "shard index out of range");
  if (start) *start = d->start[shard];
  if (len) *len = d->len[shard];
  if (state) *state = d->state[shard];
  if (owner) *owner = d->owner[shard];
  return ANTDT_OK;
}

int antdt_dds_counts(const antdt_dds* d, int64_t* todo, int64_t* doing, int64_t* done) {
  if (!d) return bad("antdt_dds_counts", "null argument");
  int64_t c[3] = {0, 0, 0};
  for (int32_t s : d->state) ++c[s];
  if (todo) *todo = c[ANTDT_SHARD_TODO];
  if (doing) *doing = c[ANTDT_SHARD_DOING];
  if (done) *done = c[ANTDT_SHARD_DONE];
  return ANTDT_OK;
}

int antdt_simulate_bsp(const antdt_sim_config* cfg, antdt_sim_result* res, int64_t* final_sizes) {
  const char* fn = "antdt_simulate_bsp";
  if (!cfg || !res) return bad(fn, "null argument");
  const antdt_sim_config& c = *cfg;
  const int n = c.n;
  if (n < 1 || n > ANTDT_MAX_SHARDS) return bad(fn, "number of workers out of range");
  if (c.B < n || c.N < 1) return bad(fn, "B >= n and N >= 1 required");
  if (!c.t0 || !c.v) return bad(fn, "null t0 or v");
  for (int i = 0; i < n; ++i)
    if (!(c.v[i] > 0.0) || !isfinite(c.v[i]) || !(c.t0[i] >= 0.0) || !isfinite(c.t0[i]) ||
        (c.persistent_delay && !(c.persistent_delay[i] >= 0.0)))
      return bad(fn, "t0 >= 0, v > 0 and delays >= 0 required");
  if (c.policy < ANTDT_POLICY_BSP || c.policy > ANTDT_POLICY_ANTDT_ND) return bad(fn, "unknown policy");
  if (!(c.period > 0.0) || !(c.duration >= 0.0) || !(c.prob >= 0.0) || !(c.decide_every > 0.0) || !(c.lambda >= 1.0) ||
      !(c.L_trans > 0.0) || !(c.L_per > 0.0) || !(c.restart_cost >= 0.0) || c.backup_b < 0 || c.backup_b >= n ||
      c.max_iterations < 1)
    return bad(fn, "parameter out of range");

  std::vector<double> pers(n, 0.0), absent_until(n, 0.0);
  if (c.persistent_delay)
    for (int i = 0; i < n; ++i) pers[i] = c.persistent_delay[i];
  std::vector<std::deque<Rec>> hist(n);
  std::vector<int> present, present_prev;
  std::vector<int64_t> sizes(n, 0), split;
  std::vector<double> T(n, 0.0), speeds;
  double t = 0.0, max_bpt = 0.0, sum_bpt = 0.0;
  int64_t processed = 0, iterations = 0;
  int32_t adjust_actions = 0, kills = 0;
  double next_decision = c.decide_every;
  const double keep = std::max(c.L_trans, c.L_per);

  auto window_mean = [&](int i, double L, int what, double* out) -> bool {
    double acc = 0.0;
    int64_t cnt = 0;
    for (const Rec& r : hist[i])
      if (r.t_end > t - L) {
        acc = acc + (what == 0 ? r.T : (double)r.b / r.T);
        ++cnt;
      }
    if (!cnt) return false;
    *out = acc / (double)cnt;
    return true;
  };

  while (processed < c.N && iterations < c.max_iterations) {
    present.clear();
    for (int i = 0; i < n; ++i)
      if (t >= absent_until[i]) present.push_back(i);
    if (present != present_prev) {  // membership changed: equal split among those present
      const int64_t m = (int64_t)present.size(), q = c.B / m, r = c.B % m;
      std::fill(sizes.begin(), sizes.end(), 0);
      for (int64_t j = 0; j < m; ++j) sizes[present[j]] = q + (j < r ? 1 : 0);
      present_prev = present;
    }
    const int64_t window = (int64_t)floor(t / c.period);
    const bool in_burst = (t - (double)window * c.period) < c.duration;
    for (int i : present) {
      double delay = pers[i];
      if (c.prob > 0.0 && in_burst && disturbed(c.seed, window, i, c.prob)) delay = delay + c.sleep_duration * c.intensity;
      T[i] = c.t0[i] + (double)sizes[i] / c.v[i] + delay;
    }
    double bpt;
    int64_t done;
    if (c.policy == ANTDT_POLICY_BACKUP_WORKERS && c.backup_b > 0) {
      std::vector<int> order = present;
      std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return T[a] < T[b] || (T[a] == T[b] && a < b); });
      const size_t inc = std::max<int64_t>((int64_t)present.size() - c.backup_b, 1);
      bpt = T[order[inc - 1]];
      done = 0;
      for (size_t j = 0; j < inc; ++j) done += sizes[order[j]];
    } else {
      bpt = T[present[0]];
      for (int i : present) bpt = std::max(bpt, T[i]);
      done = c.B;
    }
    const double step = bpt + c.t_server;
    t = t + step;
    processed += done;
    ++iterations;
    max_bpt = std::max(max_bpt, bpt);
    sum_bpt = sum_bpt + bpt;
    for (int i : present) {
      hist[i].push_back({t, sizes[i], T[i]});
      while (!hist[i].empty() && hist[i].front().t_end <= t - keep) hist[i].pop_front();
    }
    if (t < next_decision) continue;
    while (next_decision <= t) next_decision = next_decision + c.decide_every;
    if (c.policy != ANTDT_POLICY_ADJUST_BS && c.policy != ANTDT_POLICY_ANTDT_ND) continue;

    bool killed = false;
    if (c.policy == ANTDT_POLICY_ANTDT_ND && present.size() > 1) {
      std::vector<double> per(n, 0.0);
      bool ok = true;
      for (int i : present) ok = window_mean(i, c.L_per, 0, &per[i]) && ok;
      if (ok) {
        double mean = 0.0;
        for (int i : present) mean = mean + per[i];
        mean = mean / (double)present.size();
        int worst = present[0];
        for (int i : present)
          if (per[i] > per[worst]) worst = i;  // ties: lowest index
        if (per[worst] >= c.lambda * mean) {
          absent_until[worst] = t + c.restart_cost;
          pers[worst] = 0.0;
          hist[worst].clear();
          ++kills;
          killed = true;
        }
      }
    }
    if (killed) continue;  // the next iteration re-splits among those present
    std::vector<double> tr(n, 0.0);
    bool ok = true;
    for (int i : present) ok = window_mean(i, c.L_trans, 0, &tr[i]) && ok;
    if (!ok) continue;
    double mean = 0.0, hi = tr[present[0]], lo = tr[present[0]];
    for (int i : present) {
      mean = mean + tr[i];
      hi = std::max(hi, tr[i]);
      lo = std::min(lo, tr[i]);
    }
    mean = mean / (double)present.size();
    if (hi >= c.lambda * mean || lo * c.lambda <= mean) {
      speeds.assign(present.size(), 0.0);
      bool pos = true;
      for (size_t j = 0; j < present.size(); ++j) pos = window_mean(present[j], c.L_trans, 1, &speeds[j]) && speeds[j] > 0.0 && pos;
      if (pos) {
        split_by_speed(c.B, speeds, split);
        for (size_t j = 0; j < present.size(); ++j) sizes[present[j]] = split[j];
        ++adjust_actions;
      }
    }
  }
  res->jct = t;
  res->iterations = iterations;
  res->processed = processed;
  res->adjust_actions = adjust_actions;
  res->kills = kills;
  res->max_bpt = max_bpt;
  res->sum_bpt = sum_bpt;
  if (final_sizes)
    for (int i = 0; i < n; ++i) final_sizes[i] = sizes[i];
  return ANTDT_OK;
}

}  // extern "C"
