// Host-side placement scheduler (paper Sections 3.3 and 3.4): balance ratio (Eq. 6), the cost of a
// step (Eq. 5 from Eq. 7 and optionally Eq. 9), the Policy Maker (Alg. 2), one pass of the
// Scheduler (Alg. 1) with the Expand / Shrink / Migrate primitives, and the export of a placement
// as the router's table.  Plain C++ on host memory; every decision is integer arithmetic.
//
// The cost of a placement depends on the slots only through cnt[e][g], the number of vExperts of
// expert e on GPU g: slots are numbered GPU by GPU, so the first (I_e mod n_e) vExperts of e in
// ascending slot id -- the ones that take an extra token -- are a prefix of its GPUs in ascending
// GPU id.  A candidate modification therefore costs O(G) to evaluate: only the rows of the one or
// two experts it touches change.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "flexmoe.h"
#include "flexmoe_scheduler.h"

namespace {

typedef __int128 wide_t;

struct Cluster {
  int E = 0, G = 0, S = 0, V = 0;
  const int64_t* tokens = nullptr;
  int64_t token_cost = 0;
  const int64_t* sync = nullptr;          // [G+1] or null
  std::vector<int32_t> owner;             // [V]
  std::vector<int32_t> cnt;               // [E][G]
  std::vector<int32_t> n;                 // [E]
  std::vector<int64_t> time;              // [G]  Eq. 5's sum for each GPU under `owner`

  int32_t* row(int e) { return cnt.data() + (size_t)e * G; }
  const int32_t* row(int e) const { return cnt.data() + (size_t)e * G; }

  // out[g] += sign * (tokens of e computed on g), for an expert with r[g] vExperts on GPU g
  void add_tokens(int e, const int32_t* r, int64_t sign, int64_t* out) const {
    int64_t n_e = 0;
    for (int g = 0; g < G; ++g) n_e += r[g];
    if (n_e == 0) return;
    const int64_t q = tokens[e] / n_e, m = tokens[e] % n_e;
    int64_t before = 0;                   // vExperts of e on lower GPUs
    for (int g = 0; g < G; ++g) {
      const int64_t c = r[g];
      if (c == 0) continue;
      const int64_t extra = std::min(c, std::max<int64_t>(m - before, 0));
      out[g] += sign * (q * c + extra);
      before += c;
    }
  }

  // out[g] += sign * (T_C + T_Sync of e on g)
  void add_terms(int e, const int32_t* r, int64_t sign, int64_t* out) const {
    int64_t n_e = 0;
    int spread = 0;
    for (int g = 0; g < G; ++g) {
      n_e += r[g];
      spread += r[g] > 0;
    }
    if (n_e == 0) return;
    const int64_t q = tokens[e] / n_e, m = tokens[e] % n_e;
    const int64_t sync_e = sync ? sync[spread] : 0;
    int64_t before = 0;
    for (int g = 0; g < G; ++g) {
      const int64_t c = r[g];
      if (c == 0) continue;
      const int64_t extra = std::min(c, std::max<int64_t>(m - before, 0));
      out[g] += sign * ((q * c + extra) * token_cost + sync_e);
      before += c;
    }
  }

  void recount() {
    std::fill(cnt.begin(), cnt.end(), 0);
    std::fill(n.begin(), n.end(), 0);
    for (int s = 0; s < V; ++s)
      if (owner[s] != FLEXMOE_SLOT_FREE) {
        ++row(owner[s])[s / S];
        ++n[owner[s]];
      }
    std::fill(time.begin(), time.end(), 0);
    for (int e = 0; e < E; ++e) add_terms(e, row(e), +1, time.data());
  }

  int64_t cost() const { return *std::max_element(time.begin(), time.end()); }

  void gpu_loads(int64_t* load) const {
    std::fill(load, load + G, 0);
    for (int e = 0; e < E; ++e) add_tokens(e, row(e), +1, load);
  }

  double balance() const {
    std::vector<int64_t> load(G);
    gpu_loads(load.data());
    int64_t total = 0, worst = 0;
    for (int g = 0; g < G; ++g) {
      total += load[g];
      worst = std::max(worst, load[g]);
    }
    if (total == 0) return 1.0;
    return (double)(worst * G) / (double)total;     // both exact below 2^53 (checked on entry)
  }
};

int init_cluster(Cluster& c, const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                 int64_t token_cost, const int64_t* sync_cost) {
  if (!tokens || !slot_owner) return FLEXMOE_INVALID_ARG;
  if (E < 1 || E > FLEXMOE_MAX_EXPERTS || G < 1 || S < 1) return FLEXMOE_INVALID_ARG;
  if ((int64_t)G * S > FLEXMOE_MAX_SLOTS) return FLEXMOE_INVALID_ARG;
  if (token_cost < 0) return FLEXMOE_INVALID_ARG;
  const wide_t limit = (wide_t)1 << 62;
  wide_t total = 0;
  for (int e = 0; e < E; ++e) {
    if (tokens[e] < 0) return FLEXMOE_INVALID_ARG;
    total += tokens[e];
  }
  if (total * G >= ((wide_t)1 << 53)) return FLEXMOE_INVALID_ARG;
  wide_t worst = total * token_cost;
  if (sync_cost) {
    int64_t top = 0;
    for (int m = 0; m <= G; ++m) {
      if (sync_cost[m] < 0) return FLEXMOE_INVALID_ARG;
      top = std::max(top, sync_cost[m]);
    }
    worst += (wide_t)top * E;
  }
  if (worst >= limit) return FLEXMOE_INVALID_ARG;
  const int V = G * S;
  std::vector<int32_t> have(E, 0);
  for (int s = 0; s < V; ++s) {
    const int32_t o = slot_owner[s];
    if (o < FLEXMOE_SLOT_FREE || o >= E) return FLEXMOE_BAD_PLACEMENT;
    if (o >= 0) have[o] = 1;
  }
  for (int e = 0; e < E; ++e)
    if (!have[e]) return FLEXMOE_BAD_PLACEMENT;
  c.E = E; c.G = G; c.S = S; c.V = V;
  c.tokens = tokens; c.token_cost = token_cost; c.sync = sync_cost;
  c.owner.assign(slot_owner, slot_owner + V);
  c.cnt.assign((size_t)E * G, 0);
  c.n.assign(E, 0);
  c.time.assign(G, 0);
  c.recount();
  return FLEXMOE_OK;
}

// cap_a > cap_b as exact fractions
inline bool cap_greater(int64_t Ia, int32_t na, int64_t Ib, int32_t nb) { return (wide_t)Ia * nb > (wide_t)Ib * na; }

struct Plan {
  bool has = false;
  int32_t e0 = -1, source = -1, target = -1, e1 = -1, released = -1;
  int64_t t0 = 0, t1 = 0;
};

// Alg. 2
Plan make_plan(Cluster& c) {
  Plan p;
  p.t0 = c.cost();
  int e0 = 0;
  for (int e = 1; e < c.E; ++e)
    if (cap_greater(c.tokens[e], c.n[e], c.tokens[e0], c.n[e0])) e0 = e;
  int e1 = -1;
  for (int e = 0; e < c.E; ++e) {
    if (c.n[e] < 2) continue;
    if (e1 < 0 || cap_greater(c.tokens[e1], c.n[e1], c.tokens[e], c.n[e])) e1 = e;
  }
  if (e1 < 0 || e1 == e0) return p;

  const int G = c.G, S = c.S;
  std::vector<int32_t> lowest_free(G, -1);
  for (int s = c.V - 1; s >= 0; --s)
    if (c.owner[s] == FLEXMOE_SLOT_FREE) lowest_free[s / S] = s;
  // every GPU's time without the two experts; candidates add their new rows back
  std::vector<int64_t> base(c.time), trial(G);
  c.add_terms(e0, c.row(e0), -1, base.data());
  c.add_terms(e1, c.row(e1), -1, base.data());
  int32_t* r0 = c.row(e0);
  int32_t* r1 = c.row(e1);

  bool found = false;
  int64_t best = 0;
  auto consider = [&](int released, int target) {
    const int gr = released / S, gt = target / S;
    --r1[gr];
    ++r0[gt];
    trial = base;
    c.add_terms(e0, r0, +1, trial.data());
    c.add_terms(e1, r1, +1, trial.data());
    ++r1[gr];
    --r0[gt];
    const int64_t t1 = *std::max_element(trial.begin(), trial.end());
    if (!found || t1 < best) {
      found = true;
      best = t1;
      p.released = released;
      p.target = target;
    }
  };
  for (int released = 0; released < c.V; ++released) {
    if (c.owner[released] != e1) continue;
    const int gr = released / S;
    for (int g = 0; g < G; ++g) {          // targets in ascending slot id
      if (g != gr) {
        if (lowest_free[g] >= 0) consider(released, lowest_free[g]);
      } else {
        if (lowest_free[g] >= 0 && lowest_free[g] < released) consider(released, lowest_free[g]);
        consider(released, released);
      }
    }
  }
  if (!found || best >= p.t0) return p;
  p.has = true;
  p.e0 = e0;
  p.e1 = e1;
  p.t1 = best;
  const int gt = p.target / S;
  for (int s = 0; s < c.V && p.source < 0; ++s)
    if (c.owner[s] == e0 && s / S == gt) p.source = s;
  for (int s = 0; s < c.V && p.source < 0; ++s)
    if (c.owner[s] == e0) p.source = s;
  return p;
}

struct Exchange {
  bool has = false;
  int32_t a = -1, b = -1;
  int64_t t0 = 0, t1 = 0;
};

// Migrate: the best exchange that takes an expert off a GPU where it holds a single vExpert
Exchange make_exchange(Cluster& c) {
  Exchange x;
  x.t0 = c.cost();
  const int G = c.G, S = c.S;
  std::vector<int64_t> without_e(G), moved_e(G), trial(G);
  bool found = false;
  int64_t best = 0;
  for (int a = 0; a < c.V; ++a) {
    const int e = c.owner[a];
    if (e == FLEXMOE_SLOT_FREE) continue;
    const int ga = a / S;
    int32_t* re = c.row(e);
    if (re[ga] != 1) continue;
    without_e = c.time;
    c.add_terms(e, re, -1, without_e.data());
    for (int gb = 0; gb < G; ++gb) {
      if (gb == ga || re[gb] == 0) continue;
      --re[ga];
      ++re[gb];
      moved_e = without_e;
      c.add_terms(e, re, +1, moved_e.data());
      ++re[ga];
      --re[gb];
      for (int b = gb * S; b < (gb + 1) * S; ++b) {
        const int other = c.owner[b];
        if (other == e) continue;
        trial = moved_e;
        if (other != FLEXMOE_SLOT_FREE) {
          int32_t* ro = c.row(other);
          c.add_terms(other, ro, -1, trial.data());
          --ro[gb];
          ++ro[ga];
          c.add_terms(other, ro, +1, trial.data());
          ++ro[gb];
          --ro[ga];
        }
        const int64_t t1 = *std::max_element(trial.begin(), trial.end());
        if (!found || t1 < best) {
          found = true;
          best = t1;
          x.a = a;
          x.b = b;
        }
      }
    }
  }
  if (!found || best >= x.t0) return x;
  x.has = true;
  x.t1 = best;
  return x;
}

}  // namespace

extern "C" {

int flexmoe_balance_ratio(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                          double* ratio, int64_t* gpu_load) {
  if (!ratio) return FLEXMOE_INVALID_ARG;
  Cluster c;
  const int st = init_cluster(c, tokens, slot_owner, E, G, S, 0, nullptr);
  if (st != FLEXMOE_OK) return st;
  *ratio = c.balance();
  if (gpu_load) c.gpu_loads(gpu_load);
  return FLEXMOE_OK;
}

int flexmoe_step_cost(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                      int64_t token_cost, const int64_t* sync_cost, int64_t* cost) {
  if (!cost) return FLEXMOE_INVALID_ARG;
  Cluster c;
  const int st = init_cluster(c, tokens, slot_owner, E, G, S, token_cost, sync_cost);
  if (st != FLEXMOE_OK) return st;
  *cost = c.cost();
  return FLEXMOE_OK;
}

int flexmoe_make_scheduling_plan(const int64_t* tokens, const int32_t* slot_owner, int E, int G, int S,
                                 int64_t token_cost, const int64_t* sync_cost,
                                 int32_t plan[5], int64_t t[2], int* has_plan) {
  if (!plan || !t || !has_plan) return FLEXMOE_INVALID_ARG;
  Cluster c;
  const int st = init_cluster(c, tokens, slot_owner, E, G, S, token_cost, sync_cost);
  if (st != FLEXMOE_OK) return st;
  const Plan p = make_plan(c);
  *has_plan = p.has ? 1 : 0;
  plan[0] = p.has ? p.e0 : -1;
  plan[1] = p.has ? p.source : -1;
  plan[2] = p.has ? p.target : -1;
  plan[3] = p.has ? p.e1 : -1;
  plan[4] = p.has ? p.released : -1;
  t[0] = p.t0;
  t[1] = p.has ? p.t1 : p.t0;
  return FLEXMOE_OK;
}

int flexmoe_schedule(const int64_t* tokens, int32_t* slot_owner, int E, int G, int S,
                     int64_t token_cost, const int64_t* sync_cost, double threshold, int max_ops,
                     int32_t* ops, int* n_ops, double* ratio_before, double* ratio_after) {
  if (!n_ops || !ratio_before || !ratio_after || max_ops < 0 || (max_ops > 0 && !ops)) return FLEXMOE_INVALID_ARG;
  if (!(threshold == threshold)) return FLEXMOE_INVALID_ARG;      // NaN
  Cluster c;
  const int st = init_cluster(c, tokens, slot_owner, E, G, S, token_cost, sync_cost);
  if (st != FLEXMOE_OK) return st;
  int count = 0;
  auto emit = [&](int kind, int e, int a, int b) {
    int32_t* o = ops + (size_t)count * 4;
    o[0] = kind; o[1] = e; o[2] = a; o[3] = b;
    ++count;
  };
  const double before = c.balance();
  double ratio = before;
  while (ratio > threshold && count + 2 <= max_ops) {
    const Plan p = make_plan(c);
    if (!p.has) break;
    emit(FLEXMOE_SHRINK, p.e1, p.released, -1);
    emit(FLEXMOE_EXPAND, p.e0, p.source, p.target);
    c.owner[p.released] = FLEXMOE_SLOT_FREE;
    c.owner[p.target] = p.e0;
    c.recount();
    ratio = c.balance();
  }
  if (count + 1 <= max_ops) {
    const Exchange x = make_exchange(c);
    if (x.has) {
      emit(FLEXMOE_MIGRATE, c.owner[x.a], x.a, x.b);
      std::swap(c.owner[x.a], c.owner[x.b]);
      c.recount();
      ratio = c.balance();
    }
  }
  std::copy(c.owner.begin(), c.owner.end(), slot_owner);
  *n_ops = count;
  *ratio_before = before;
  *ratio_after = ratio;
  return FLEXMOE_OK;
}

int flexmoe_placement_table(const int32_t* slot_owner, int E, int n_slots,
                            int32_t* rep_off, int32_t* rep_ids, int* V) {
  if (!slot_owner || !rep_off || !rep_ids || !V) return FLEXMOE_INVALID_ARG;
  if (E < 1 || E > FLEXMOE_MAX_EXPERTS || n_slots < 1 || n_slots > FLEXMOE_MAX_SLOTS) return FLEXMOE_INVALID_ARG;
  std::vector<int32_t> n(E, 0);
  for (int s = 0; s < n_slots; ++s) {
    const int32_t o = slot_owner[s];
    if (o < FLEXMOE_SLOT_FREE || o >= E) return FLEXMOE_BAD_PLACEMENT;
    if (o >= 0) ++n[o];
  }
  for (int e = 0; e < E; ++e)
    if (n[e] == 0) return FLEXMOE_BAD_PLACEMENT;
  rep_off[0] = 0;
  for (int e = 0; e < E; ++e) rep_off[e + 1] = rep_off[e] + n[e];
  std::vector<int32_t> fill(rep_off, rep_off + E);
  int32_t vid = 0;
  for (int s = 0; s < n_slots; ++s)
    if (slot_owner[s] != FLEXMOE_SLOT_FREE) rep_ids[fill[slot_owner[s]]++] = vid++;
  *V = vid;
  return FLEXMOE_OK;
}

}  // extern "C"
