// Host side of the method around the kernels: the kernel analyzer's data-dependency graph
// (Sec. 3.1, "Data dependency analysis") and the policy planner (Sec. 3.2).  No device code.
//
// Dependency graph: kernels are visited in execution order against a registry of the last
// writer of every byte (an ordered map of disjoint intervals); a read adds an edge from the
// most recent writer of each piece it overlaps, a kernel never depends on itself, edges between
// the same two kernels are merged.  The list is run for two iterations; a read of the second
// iteration that is served by a write of the first is a cross-iteration dependency (the KV
// cache pattern), reported with its flag set.
//
// Planner: both objectives of Sec. 3.2 over placements x[k] in G,
//   T_g = sum_k t[k][g] [x_k = g],  M_g = sum over edges (i,j) cut into g of (l[u][g] + d_ij / bw[u][g]),
//   throughput:  min max_g max(T_g, M_g)        latency:  min sum_g T_g + sum_g M_g.
// The paper hands the linearised MILP to a commercial solver; here the latency objective is
// solved exactly by dynamic programming over the frontier of kernels whose outputs are still
// needed (a decoder stack keeps that frontier at two or three kernels, so 500 kernels take
// microseconds), and the throughput objective by depth-first branch and bound in execution order
// (T_g and M_g only grow along a branch, so max_g max(T_g, M_g) and the average-load bound
// prune), exact unless the node limit stops it.
#include <algorithm>
#include <cmath>
#include <limits>
#include <map>
#include <tuple>
#include <unordered_map>
#include <utility>
#include <vector>

#include "common.hpp"

namespace ts {
namespace {

struct WriteInst {       // one write access of one kernel launch
  int writer, iter;
  uint64_t bytes;        // bytes that write actually touched inside its hull
};
struct Piece {           // registry entry: bytes [lo, hi) were last written by write instance `wid`
  uint64_t hi;
  int wid;
};

using Registry = std::map<uint64_t, Piece>;   // key = lo

void registry_write(Registry& reg, uint64_t lo, uint64_t hi, int wid) {
  if (hi <= lo) return;
  auto it = reg.lower_bound(lo);
  if (it != reg.begin()) {
    auto pv = std::prev(it);
    if (pv->second.hi > lo) {                       // split the piece that straddles lo
      Piece tail = pv->second;
      pv->second.hi = lo;
      if (tail.hi > hi) reg[hi] = tail;             // ... and survives beyond hi
    }
  }
  while (it != reg.end() && it->first < hi) {
    if (it->second.hi > hi) {                       // keep the part beyond hi
      Piece tail = it->second;
      reg.erase(it);
      reg[hi] = tail;
      break;
    }
    it = reg.erase(it);
  }
  reg[lo] = Piece{hi, wid};
}

struct EdgeKey {
  int src, dst, cross;
  bool operator<(const EdgeKey& o) const {
    if (cross != o.cross) return cross < o.cross;
    if (src != o.src) return src < o.src;
    return dst < o.dst;
  }
};

int ddg_build_impl(const ts_kernel_io* ks, int n, std::vector<ts_ddg_edge>& out) {
  Registry reg;
  std::vector<WriteInst> inst;
  std::map<EdgeKey, uint64_t> acc;
  std::map<int, uint64_t> ov;                       // write instance -> bytes of this read it still owns
  for (int iter = 0; iter < 2; ++iter) {
    for (int k = 0; k < n; ++k) {
      for (int r = 0; r < ks[k].n_reads; ++r) {
        if (iter == 0) break;                       // the first iteration only fills the registry
        const ts_access& a = ks[k].reads[r];
        const uint64_t lo = a.addr + (uint64_t)(a.iter_advance * iter), hi = lo + a.extent;
        if (hi <= lo) continue;
        ov.clear();
        auto it = reg.upper_bound(lo);
        if (it != reg.begin()) --it;
        for (; it != reg.end() && it->first < hi; ++it) {
          const uint64_t a0 = std::max(lo, it->first), a1 = std::min(hi, it->second.hi);
          if (a1 > a0) ov[it->second.wid] += a1 - a0;
        }
        for (const auto& kv : ov) {
          const WriteInst& w = inst[kv.first];
          if (w.iter == iter && w.writer == k) continue;
          const uint64_t flow = std::min(std::min(kv.second, w.bytes), (uint64_t)a.bytes);
          acc[EdgeKey{w.writer, k, w.iter == iter ? 0 : 1}] += flow;
        }
      }
      for (int w = 0; w < ks[k].n_writes; ++w) {
        const ts_access& a = ks[k].writes[w];
        const uint64_t lo = a.addr + (uint64_t)(a.iter_advance * iter);
        inst.push_back(WriteInst{k, iter, a.bytes});
        registry_write(reg, lo, lo + a.extent, (int)inst.size() - 1);
      }
    }
  }
  out.clear();
  for (const auto& kv : acc) {
    ts_ddg_edge e{};
    e.src = kv.first.src;
    e.dst = kv.first.dst;
    e.bytes = kv.second;
    e.cross_iteration = kv.first.cross;
    out.push_back(e);
  }
  return TS_OK;
}

// ---------------------------------------------------------------------------- planner
struct Problem {
  int K, G;
  const double* t;
  std::vector<std::vector<std::pair<int, double>>> in;   // per kernel: (producer, bytes) of intra-iteration edges
  const double *bw, *lat;
  double cost(int u, int g, double d) const { return lat[u * G + g] + d / bw[u * G + g]; }
};

void evaluate(const Problem& p, const int32_t* place, std::vector<double>& T, std::vector<double>& M) {
  T.assign(p.G, 0.0);
  M.assign(p.G, 0.0);
  for (int k = 0; k < p.K; ++k) {
    const int g = place[k];
    T[g] += p.t[k * p.G + g];
    for (const auto& e : p.in[k]) {
      const int u = place[e.first];
      if (u != g) M[g] += p.cost(u, g, e.second);
    }
  }
}

// Latency objective: exact frontier DP.  State = placement of the kernels that still have a consumer ahead.
bool plan_latency_dp(const Problem& p, std::vector<int32_t>& best_place, double& best) {
  const int K = p.K, G = p.G;
  std::vector<int> last_use(K, -1);
  for (int k = 0; k < K; ++k)
    for (const auto& e : p.in[k]) last_use[e.first] = std::max(last_use[e.first], k);
  int bits = 1;
  while ((1 << bits) < G) ++bits;
  // live list before kernel k, in ascending kernel order
  std::vector<std::vector<int>> live(K + 1);
  for (int k = 0; k < K; ++k) {
    live[k + 1] = live[k];
    live[k + 1].erase(std::remove_if(live[k + 1].begin(), live[k + 1].end(), [&](int i) { return last_use[i] <= k; }),
                      live[k + 1].end());
    if (last_use[k] > k) live[k + 1].push_back(k);
    if ((int)live[k + 1].size() * bits > 60) return false;   // frontier too wide for this encoding
  }
  struct Entry { double cost; uint64_t prev; int g; };
  std::vector<std::unordered_map<uint64_t, Entry>> layers(K + 1);
  layers[0][0] = Entry{0.0, 0, -1};
  for (int k = 0; k < K; ++k) {
    const auto& lv = live[k];
    const auto& nx = live[k + 1];
    for (const auto& kv : layers[k]) {
      const uint64_t st = kv.first;
      auto placed = [&](int i) {
        const int pos = (int)(std::find(lv.begin(), lv.end(), i) - lv.begin());
        return (int)((st >> (pos * bits)) & ((1u << bits) - 1));
      };
      for (int g = 0; g < G; ++g) {
        double c = kv.second.cost + p.t[k * G + g];
        for (const auto& e : p.in[k]) {
          const int u = placed(e.first);
          if (u != g) c += p.cost(u, g, e.second);
        }
        uint64_t ns = 0;
        for (size_t q = 0; q < nx.size(); ++q) {
          const int pl = nx[q] == k ? g : placed(nx[q]);
          ns |= (uint64_t)pl << (q * bits);
        }
        auto it = layers[k + 1].find(ns);
        if (it == layers[k + 1].end() || c < it->second.cost) layers[k + 1][ns] = Entry{c, st, g};
      }
    }
  }
  best = std::numeric_limits<double>::infinity();
  uint64_t st = 0;
  for (const auto& kv : layers[K])
    if (kv.second.cost < best) { best = kv.second.cost; st = kv.first; }
  best_place.assign(K, 0);
  for (int k = K; k > 0; --k) {
    const Entry& e = layers[k].at(st);
    best_place[k - 1] = e.g;
    st = e.prev;
  }
  return true;
}

// Incumbent for the search: the best split of the execution order into G contiguous stages (stage g on GPU g,
// stages may be empty), by dynamic programming with every incoming edge priced as if it came from the
// previous GPU.  Only a starting point: the caller evaluates it exactly.
void contiguous_seed(const Problem& p, std::vector<int32_t>& place) {
  const int K = p.K, G = p.G;
  const double inf = std::numeric_limits<double>::infinity();
  std::vector<std::vector<double>> f(G + 1, std::vector<double>(K + 1, inf));
  std::vector<std::vector<int>> from(G + 1, std::vector<int>(K + 1, 0));
  f[0][0] = 0.0;
  for (int g = 1; g <= G; ++g) {
    const int dev = g - 1, src = g >= 2 ? g - 2 : 0;
    for (int a = 0; a <= K; ++a) {
      if (f[g - 1][a] == inf) continue;
      double T = 0.0, M = 0.0;
      for (int b = a; b <= K; ++b) {
        if (b > a) {
          const int k = b - 1;
          T += p.t[k * G + dev];
          if (dev != src)
            for (const auto& e : p.in[k])
              if (e.first < a) M += p.cost(src, dev, e.second);
        }
        const double c = std::max(f[g - 1][a], std::max(T, M));
        if (c < f[g][b]) { f[g][b] = c; from[g][b] = a; }
      }
    }
  }
  place.assign(K, 0);
  int b = K;
  for (int g = G; g >= 1; --g) {
    const int a = from[g][b];
    for (int k = a; k < b; ++k) place[k] = g - 1;
    b = a;
  }
}

struct BnB {
  const Problem& p;
  int objective;
  int64_t node_limit, nodes = 0;
  bool exhausted = false;
  // stop as soon as the incumbent is within rel_gap of `root_lb`, a lower bound of the optimum (0: never)
  double rel_gap = 0.0, root_lb = 0.0;
  bool within_gap = false;
  bool close_enough() const { return rel_gap > 0.0 && best <= root_lb * (1.0 + rel_gap); }
  std::vector<double> T, M, rem_min;          // rem_min[k] = sum_{j >= k} min_g t[j][g]
  std::vector<int32_t> place, best_place;
  double best = std::numeric_limits<double>::infinity();

  double bound(int k) const {                 // lower bound of any completion with kernels < k placed
    if (objective == TS_PLAN_LATENCY) {
      double s = rem_min[k];
      for (int g = 0; g < p.G; ++g) s += T[g] + M[g];
      return s;
    }
    double mx = 0.0, sum = rem_min[k];
    for (int g = 0; g < p.G; ++g) {
      mx = std::max(mx, std::max(T[g], M[g]));
      sum += T[g];
    }
    mx = std::max(mx, sum / p.G);
    if (p.G == 2 && k < p.K) mx = std::max(mx, two_gpu_fractional(k));
    return mx;
  }
  // Two GPUs: the makespan when the remaining kernels may be split fractionally between the two (no
  // communication) bounds every integral completion from below.  Start with all of them on GPU 0 and move
  // them over in ascending order of (time on GPU 1) / (time on GPU 0) until the two loads meet.
  std::vector<int> by_ratio;                   // all kernels, ascending t[k][1] / t[k][0]
  // The same walk in O(log K): for every suffix k the kernels j >= k in ratio order with running sums of their
  // times (built once, K^2 / 2 entries per table; used up to kFracTableMax kernels, the linear walk beyond).
  // The running sums round differently from the walk, so the result is lowered by a relative 1e-13: a bound
  // only has to stay below the truth.
  static constexpr int kFracTableMax = 2048;
  std::vector<size_t> frac_begin;                      // [K+1] start of suffix k's list
  std::vector<double> frac_a, frac_b;                  // per entry: that kernel's time on GPU 0 / GPU 1
  std::vector<double> frac_sa, frac_sb, frac_sab;      // running sums up to and including the entry
  void build_fractional_tables() {
    const int K = p.K;
    if (p.G != 2 || K > kFracTableMax) return;
    frac_begin.assign(K + 1, 0);
    size_t total = 0;
    for (int k = 0; k <= K; ++k) { frac_begin[k] = total; total += (size_t)(K - k); }
    frac_a.resize(total); frac_b.resize(total); frac_sa.resize(total); frac_sb.resize(total); frac_sab.resize(total);
    std::vector<size_t> fill(frac_begin.begin(), frac_begin.end() - 1);
    for (int j : by_ratio) {
      const double a = p.t[j * 2], b = p.t[j * 2 + 1];
      for (int k = 0; k <= j; ++k) {                   // kernel j belongs to every suffix k <= j
        const size_t at = fill[k]++;
        const bool first = at == frac_begin[k];
        frac_a[at] = a; frac_b[at] = b;
        frac_sa[at] = (first ? 0.0 : frac_sa[at - 1]) + a;
        frac_sb[at] = (first ? 0.0 : frac_sb[at - 1]) + b;
        frac_sab[at] = frac_sa[at] + frac_sb[at];
      }
    }
  }
  double two_gpu_fractional(int k) const {
    double L0 = T[0] + rem0[k], L1 = T[1];
    if (L1 >= L0) return L1;
    if (!frac_begin.empty()) {
      // entry i can be moved whole (after the entries before it) iff L1 + sb[i] <= L0 - sa[i]
      const size_t lo = frac_begin[k], hi = frac_begin[k + 1];
      const double diff = L0 - L1;
      const size_t m = (size_t)(std::upper_bound(frac_sab.begin() + lo, frac_sab.begin() + hi, diff) - (frac_sab.begin() + lo));
      if (m > 0) { L0 -= frac_sa[lo + m - 1]; L1 += frac_sb[lo + m - 1]; }
      const double slack = 1.0 - 1e-13;
      if (m == hi - lo) return std::max(L0, L1) * slack;
      const double a = frac_a[lo + m], b = frac_b[lo + m];
      if (a <= 0.0) return std::max(L0, L1) * slack;   // nothing left that relieves GPU 0
      return (L1 + (L0 - L1) / (a + b) * b) * slack;   // the fraction of that kernel that makes the loads equal
    }
    for (int j : by_ratio) {
      if (j < k) continue;
      const double a = p.t[j * 2], b = p.t[j * 2 + 1];
      if (a <= 0.0) break;                     // nothing left that relieves GPU 0
      if (L1 + b <= L0 - a) { L0 -= a; L1 += b; continue; }
      const double y = (L0 - L1) / (a + b);    // fraction of kernel j that makes the loads equal
      return L1 + y * b;
    }
    return std::max(L0, L1);
  }
  std::vector<double> rem0;                    // rem0[k] = sum_{j >= k} t[j][0]
  void dfs(int k) {
    if (exhausted) return;
    if (++nodes > node_limit) { exhausted = true; return; }
    if (k == p.K) {
      const double v = bound(k);
      if (v < best) {
        best = v;
        best_place = place;
        if (close_enough()) { within_gap = true; exhausted = true; }   // good enough: unwind
      }
      return;
    }
    // children ordered by their bound
    std::vector<std::pair<double, int>> order;
    std::vector<double> dT(p.G), dM(p.G);
    for (int g = 0; g < p.G; ++g) {
      dT[g] = p.t[k * p.G + g];
      dM[g] = 0.0;
      for (const auto& e : p.in[k]) {
        const int u = place[e.first];
        if (u != g) dM[g] += p.cost(u, g, e.second);
      }
      T[g] += dT[g]; M[g] += dM[g];
      order.push_back({bound(k + 1), g});
      T[g] -= dT[g]; M[g] -= dM[g];
    }
    std::sort(order.begin(), order.end());
    for (const auto& o : order) {
      if (o.first >= best) break;
      const int g = o.second;
      const double t0 = T[g], m0 = M[g];
      T[g] += dT[g]; M[g] += dM[g];
      place[k] = g;
      dfs(k + 1);
      T[g] = t0; M[g] = m0;                    // restore exactly (no accumulated rounding)
    }
  }
};


// Two GPUs, throughput objective: fine balancing of a placement.  The search above dives in execution order and
// can only revise its late decisions, and a decoder stack repeats a handful of kernel shapes, so the loads
// (T_0, T_1) it reaches are a coarse subset of what is reachable.  This step looks at whole classes of equal
// kernels instead: a class is (current GPU, time on GPU 0, time on GPU 1); moving c kernels of a class to the
// other GPU changes the loads by c * (-a, +b) or c * (+a, -b).  The classes are cut into two halves, every
// combination of counts (0 .. a small window) is enumerated per half, and the halves are joined through the
// Pareto front of one of them: the best combinations by max(T_0, T_1) are then applied (members of a class
// are taken in the order of what the move adds to the communication terms) and evaluated exactly, communication
// included; the placement is replaced only by a strictly better one.
struct Polish {
  const Problem& p;
  std::vector<std::vector<int>> outs;                       // consumers of every kernel (the problem stores producers)

  explicit Polish(const Problem& pr) : p(pr), outs(pr.K) {
    for (int k = 0; k < p.K; ++k)
      for (const auto& e : p.in[k]) outs[e.first].push_back(k);
  }
  static double objective_of(const std::vector<double>& T, const std::vector<double>& M) {
    double v = 0.0;
    for (size_t g = 0; g < T.size(); ++g) v = std::max(v, std::max(T[g], M[g]));
    return v;
  }
  // what flipping kernel k alone adds to M_0 + M_1 under `place`
  double flip_comm_delta(const std::vector<int32_t>& place, int k) const {
    const int g = place[k], h = 1 - g;
    double d = 0.0;
    for (const auto& e : p.in[k]) {
      const int u = place[e.first];
      if (u != g) d -= p.cost(u, g, e.second);
      if (u != h) d += p.cost(u, h, e.second);
    }
    for (int j : outs[k]) {
      const int gj = place[j];
      for (const auto& e : p.in[j])
        if (e.first == k) {
          if (g != gj) d -= p.cost(g, gj, e.second);
          if (h != gj) d += p.cost(h, gj, e.second);
        }
    }
    return d;
  }
  struct Class { double a, b; std::vector<int> on0, on1; int lo = 0, hi = 0; };   // count range: lo <= 0 <= hi
  struct Combo { double d0, d1; uint32_t code; };

  bool run(std::vector<int32_t>& place, double& value) const {
    if (p.G != 2 || p.K < 2) return false;
    std::vector<double> T, M;
    evaluate(p, place.data(), T, M);
    // classes of kernels with equal times; a count c > 0 moves c members from GPU 0 to GPU 1, c < 0 the other way:
    // the loads change by (-c a, +c b) either way
    std::map<std::pair<double, double>, int> index;
    std::vector<Class> cls;
    for (int k = 0; k < p.K; ++k) {
      const auto key = std::make_pair(p.t[k * 2], p.t[k * 2 + 1]);
      auto it = index.find(key);
      if (it == index.end()) {
        it = index.emplace(key, (int)cls.size()).first;
        cls.push_back(Class{key.first, key.second, {}, {}});
      }
      (place[k] == 0 ? cls[it->second].on0 : cls[it->second].on1).push_back(k);
    }
    std::vector<double> cheapest(cls.size(), std::numeric_limits<double>::infinity());
    for (size_t c = 0; c < cls.size(); ++c) {
      for (auto* m : {&cls[c].on0, &cls[c].on1}) {
        std::vector<std::pair<double, int>> by_cost;
        for (int k : *m) by_cost.push_back({flip_comm_delta(place, k), k});
        std::sort(by_cost.begin(), by_cost.end());
        for (size_t i = 0; i < m->size(); ++i) (*m)[i] = by_cost[i].second;
        if (!by_cost.empty()) cheapest[c] = std::min(cheapest[c], by_cost[0].first);
      }
    }
    // digits: classes in the order of their cheapest move, counts in a window around 0 sized so that each of the
    // two halves has at most 2^16 combinations
    std::vector<int> order(cls.size());
    for (size_t c = 0; c < cls.size(); ++c) order[c] = (int)c;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return cheapest[x] < cheapest[y]; });
    const size_t cap = (size_t)1 << 16;
    const size_t per_half = (cls.size() + 1) / 2;
    int window = 1;
    while (window < 31 && std::pow((double)(2 * (window + 1) + 1), (double)std::min<size_t>(per_half, 16)) <= (double)cap) ++window;
    std::vector<int> half[2];
    std::vector<int> radix[2];
    size_t prod[2] = {1, 1};
    for (int c : order) {
      if (cls[c].a <= 0.0 && cls[c].b <= 0.0) continue;
      cls[c].hi = std::min<int>(window, (int)cls[c].on0.size());
      cls[c].lo = -std::min<int>(window, (int)cls[c].on1.size());
      const int r = cls[c].hi - cls[c].lo + 1;
      const int h = prod[0] <= prod[1] ? 0 : 1;
      if (r < 2 || prod[h] * (size_t)r > cap) continue;
      half[h].push_back(c);
      radix[h].push_back(r);
      prod[h] *= (size_t)r;
    }
    if (half[0].empty() && half[1].empty()) return false;
    auto enumerate = [&](int h, std::vector<Combo>& out) {
      out.assign(prod[h], Combo{0.0, 0.0, 0});
      for (size_t code = 0; code < prod[h]; ++code) {
        size_t rest = code;
        double d0 = 0.0, d1 = 0.0;
        for (size_t i = 0; i < half[h].size(); ++i) {
          const Class& c = cls[half[h][i]];
          const int cnt = c.lo + (int)(rest % (size_t)radix[h][i]);
          rest /= (size_t)radix[h][i];
          d0 -= cnt * c.a;
          d1 += cnt * c.b;
        }
        out[code] = Combo{d0, d1, (uint32_t)code};
      }
    };
    std::vector<Combo> left, right;
    enumerate(0, left);
    enumerate(1, right);
    // Pareto front of the right half: ascending d0, strictly descending d1
    std::sort(right.begin(), right.end(), [](const Combo& x, const Combo& y) { return x.d0 < y.d0 || (x.d0 == y.d0 && x.d1 < y.d1); });
    std::vector<Combo> front;
    for (const Combo& c : right)
      if (front.empty() || c.d1 < front.back().d1) front.push_back(c);
    // best joins by max(T_0, T_1)
    struct Cand { double f; uint32_t l, r; };
    std::vector<Cand> cands;
    const size_t keep = 48;
    double worst_kept = std::numeric_limits<double>::infinity();
    auto offer = [&](double f, uint32_t l, uint32_t r) {
      if (cands.size() >= keep && f >= worst_kept) return;
      cands.push_back(Cand{f, l, r});
      if (cands.size() >= 4 * keep) {
        std::nth_element(cands.begin(), cands.begin() + keep, cands.end(), [](const Cand& x, const Cand& y) { return x.f < y.f; });
        cands.resize(keep);
        worst_kept = 0.0;
        for (const Cand& c : cands) worst_kept = std::max(worst_kept, c.f);
      }
    };
    for (const Combo& l : left) {
      const double t0 = T[0] + l.d0, t1 = T[1] + l.d1;
      // first front entry where GPU 0 is at least as loaded as GPU 1 (t0 + d0 grows, t1 + d1 falls along the front)
      size_t lo = 0, hi = front.size();
      while (lo < hi) {
        const size_t mid = (lo + hi) / 2;
        if (t0 + front[mid].d0 >= t1 + front[mid].d1) hi = mid; else lo = mid + 1;
      }
      for (size_t i = (lo > 0 ? lo - 1 : 0); i < std::min(front.size(), lo + 2); ++i)
        offer(std::max(t0 + front[i].d0, t1 + front[i].d1), l.code, front[i].code);
    }
    std::sort(cands.begin(), cands.end(), [](const Cand& x, const Cand& y) { return x.f < y.f; });
    if (cands.size() > keep) cands.resize(keep);
    bool improved = false;
    const std::vector<int32_t> base = place;    // the classes and their member order refer to this placement
    std::vector<int32_t> trial;
    std::vector<double> Tt, Mt;
    for (const Cand& c : cands) {
      if (c.f >= value) break;                  // even without communication it would not beat the incumbent
      trial = base;
      const uint32_t codes[2] = {c.l, c.r};
      for (int h = 0; h < 2; ++h) {
        size_t rest = codes[h];
        for (size_t i = 0; i < half[h].size(); ++i) {
          const Class& k = cls[half[h][i]];
          const int cnt = k.lo + (int)(rest % (size_t)radix[h][i]);
          rest /= (size_t)radix[h][i];
          for (int q = 0; q < cnt; ++q) trial[k.on0[q]] = 1;
          for (int q = 0; q < -cnt; ++q) trial[k.on1[q]] = 0;
        }
      }
      evaluate(p, trial.data(), Tt, Mt);
      const double v = objective_of(Tt, Mt);
      if (v < value) { value = v; place = trial; improved = true; }
    }
    return improved;
  }
};


// ---------------------------------------------------------------------------- the layer as a kernel list
// Nodes = kernel groups ending at a kernel boundary (node i writes boundary i).  Addresses: the workspace at
// its real offsets (all layers share it, as they do at run time), then per layer the residual stream and
// the two caches in a synthetic region above it.
struct LayerNodes {
  std::vector<std::vector<ts_access>> reads, writes;
  std::vector<ts_kernel_io> io;
};

constexpr int kBoundaryBuffers = 1, kSideTables = 2;

int build_layer_nodes(const ts_layer_desc& d, int T, int B, int kv_len, int n_layers, int which, LayerNodes& out) {
  const bool moe = d.E > 0;
  const int nb = moe ? TS_NB_MOE : TS_NB_DENSE;
  const uint64_t WS = 4096;
  const uint64_t ws_bytes = (uint64_t)ts_layer_workspace_bytes(&d, T, B);
  const uint64_t xbytes = (uint64_t)T * d.H * 2;
  const uint64_t cache_bytes = (uint64_t)B * d.nkv * d.Lcap * d.d * 2;
  auto up = [](uint64_t v) { return (v + 4095) / 4096 * 4096; };
  const uint64_t EXT = WS + up(ws_bytes) + 4096;
  const uint64_t per_layer = up(xbytes) + 2 * up(cache_bytes);
  auto X = [&](int l) { return EXT + (uint64_t)l * per_layer; };                 // input of layer l = output of l-1
  auto KC = [&](int l) { return X(l) + up(xbytes); };
  auto VC = [&](int l) { return KC(l) + up(cache_bytes); };
  size_t moe_off[6] = {0, 0, 0, 0, 0, 0};
  if (moe) {
    int rc = ts_layer_moe_buffers(&d, T, B, moe_off);
    if (rc != TS_OK) return rc;
  }
  // The declared accesses of every node (the same list a GPU test holds the kernels to), once per layer shape.
  // Scratch private to a node carries nothing between nodes and is left out; the routing tables of a MoE layer
  // are data that travels outside the kernel boundaries (`kSideTables`).
  std::vector<std::vector<ts_layer_access>> decl(nb);
  for (int i = 0; i < nb; ++i) {
    int n = 0;
    int rc = ts_layer_node_accesses(&d, T, B, d.mode == TS_MODE_DECODE ? kv_len : 1, i, nullptr, 0, &n);
    if (rc != TS_OK && rc != TS_ERR_WORKSPACE) return rc;
    decl[i].resize(n);
    if (n > 0) {
      rc = ts_layer_node_accesses(&d, T, B, d.mode == TS_MODE_DECODE ? kv_len : 1, i, decl[i].data(), n, &n);
      if (rc != TS_OK) return rc;
    }
  }
  out.reads.assign((size_t)n_layers * nb, {});
  out.writes.assign((size_t)n_layers * nb, {});
  const bool bb = which & kBoundaryBuffers, st = which & kSideTables;
  for (int l = 0; l < n_layers; ++l) {
    for (int i = 0; i < nb; ++i) {
      for (const ts_layer_access& a : decl[i]) {
        if (a.kind == TS_ACC_PRIVATE) continue;
        bool side = false;
        if (moe && a.buffer == TS_BUF_WORKSPACE)
          for (size_t o : moe_off) side = side || a.offset == (uint64_t)o;
        if (side ? !st : !bb) continue;
        uint64_t base = 0;
        switch (a.buffer) {
          case TS_BUF_WORKSPACE: base = WS; break;
          case TS_BUF_X: base = X(l); break;
          case TS_BUF_OUT: base = X(l + 1); break;
          case TS_BUF_KCACHE: base = KC(l); break;
          default: base = VC(l); break;
        }
        const ts_access acc{base + a.offset, a.extent, a.bytes, a.iter_advance};
        (a.kind == TS_ACC_WRITE ? out.writes : out.reads)[(size_t)l * nb + i].push_back(acc);
      }
    }
  }
  out.io.resize(out.reads.size());
  for (size_t i = 0; i < out.io.size(); ++i)
    out.io[i] = ts_kernel_io{out.reads[i].data(), out.writes[i].data(), (int32_t)out.reads[i].size(),
                             (int32_t)out.writes[i].size()};
  return TS_OK;
}

int check_layer_args(const ts_layer_desc* desc, int T, int B, int kv_len, const char* who) {
  TS_REQUIRE(desc != nullptr, TS_ERR_INVALID_ARG, "%s: null desc", who);
  TS_REQUIRE(T >= 1 && B >= 1, TS_ERR_INVALID_ARG, "%s: T=%d B=%d must be positive", who, T, B);
  if (desc->mode == TS_MODE_DECODE) {
    TS_REQUIRE(T == B, TS_ERR_INVALID_ARG, "%s: a decode step has one token per sequence (T=%d, B=%d)", who, T, B);
    TS_REQUIRE(kv_len >= 1 && kv_len < desc->Lcap, TS_ERR_INVALID_ARG,
               "%s: kv_len=%d must leave room for the next position (Lcap=%d)", who, kv_len, desc->Lcap);
  }
  return TS_OK;
}

}  // namespace
}  // namespace ts

using namespace ts;

extern "C" {

int ts_ddg_build(const ts_kernel_io* kernels, int n_kernels, ts_ddg_edge* edges, int max_edges, int* n_edges) {
  TS_REQUIRE(n_kernels >= 0 && (kernels != nullptr || n_kernels == 0) && n_edges != nullptr && max_edges >= 0 &&
                 (edges != nullptr || max_edges == 0),
             TS_ERR_INVALID_ARG, "ts_ddg_build: null or negative argument");
  for (int k = 0; k < n_kernels; ++k)
    TS_REQUIRE(kernels[k].n_reads >= 0 && kernels[k].n_writes >= 0 && (kernels[k].reads || kernels[k].n_reads == 0) &&
                   (kernels[k].writes || kernels[k].n_writes == 0),
               TS_ERR_INVALID_ARG, "ts_ddg_build: kernel %d has a null access list", k);
  std::vector<ts_ddg_edge> out;
  ddg_build_impl(kernels, n_kernels, out);
  *n_edges = (int)out.size();
  TS_REQUIRE((int)out.size() <= max_edges, TS_ERR_WORKSPACE, "ts_ddg_build: %zu edges, room for %d", out.size(), max_edges);
  std::copy(out.begin(), out.end(), edges);
  return TS_OK;
}

int ts_layer_ddg(const ts_layer_desc* desc, int T, int B, int kv_len, int n_layers, ts_ddg_edge* edges, int max_edges,
                 int* n_edges) {
  int rc = check_layer_args(desc, T, B, kv_len, "ts_layer_ddg");
  if (rc != TS_OK) return rc;
  TS_REQUIRE(n_layers >= 1 && n_layers <= 4096 && n_edges != nullptr, TS_ERR_INVALID_ARG, "ts_layer_ddg: bad n_layers %d", n_layers);
  LayerNodes nodes;
  rc = build_layer_nodes(*desc, T, B, kv_len, n_layers, kBoundaryBuffers | kSideTables, nodes);
  if (rc != TS_OK) return rc;
  return ts_ddg_build(nodes.io.data(), (int)nodes.io.size(), edges, max_edges, n_edges);
}

const char* ts_layer_node_name(const ts_layer_desc* desc, int node) {
  static const char* dense[TS_NB_DENSE] = {"rmsnorm1", "qkv_rope_append", "attention", "o_proj_residual",
                                           "rmsnorm2", "gate_up", "swiglu", "down_residual"};
  static const char* moe[TS_NB_MOE] = {"rmsnorm1", "qkv_rope_append", "attention", "o_proj_residual", "rmsnorm2",
                                       "route_expert_gate_up", "swiglu", "expert_down", "combine_residual"};
  if (desc == nullptr || node < 0) return nullptr;
  if (desc->E > 0) return node < TS_NB_MOE ? moe[node] : nullptr;
  return node < TS_NB_DENSE ? dense[node] : nullptr;
}

int ts_layer_cut_mask(const ts_layer_desc* desc, const int32_t* placement, uint64_t* boundary_mask) {
  TS_REQUIRE(desc != nullptr && placement != nullptr && boundary_mask != nullptr, TS_ERR_INVALID_ARG,
             "ts_layer_cut_mask: null argument");
  ts_layer_desc d = *desc;
  d.mode = TS_MODE_PREFILL;               // the graph's topology does not depend on the mode or the sizes
  const int nb = d.E > 0 ? TS_NB_MOE : TS_NB_DENSE;
  uint64_t mask = 0;
  for (int which : {kBoundaryBuffers, kSideTables}) {
    LayerNodes nodes;
    int rc = build_layer_nodes(d, 1, 1, 1, 1, which, nodes);
    if (rc != TS_OK) return rc;
    std::vector<ts_ddg_edge> edges;
    ddg_build_impl(nodes.io.data(), nb, edges);
    for (const ts_ddg_edge& e : edges) {
      if (e.cross_iteration || placement[e.src] == placement[e.dst]) continue;
      TS_REQUIRE(which == kBoundaryBuffers, TS_ERR_UNSUPPORTED_SHAPE,
                 "ts_layer_cut_mask: nodes %d and %d exchange routing tables and must share a GPU", e.src, e.dst);
      mask |= 1ull << e.src;
    }
  }
  if (placement[nb - 1] != placement[nb]) mask |= 1ull << (nb - 1);
  *boundary_mask = mask;
  return TS_OK;
}

// Shared by the planner entry points: validates, searches, and reports a lower bound of the optimum.
// status: 2 = proved optimal, 1 = within rel_gap of the lower bound (proved by that bound), 0 = stopped by the node limit.
static int plan_impl(const ts_plan_problem* pr, int objective, int64_t node_limit, double rel_gap, int32_t* placement,
                     double* value, double* T_g, double* M_g, int* status, double* lower_bound, const char* who) {
  TS_REQUIRE(pr != nullptr, TS_ERR_INVALID_ARG, "%s: null problem", who);
  TS_REQUIRE(pr->n_kernels >= 1 && pr->n_gpus >= 1 && pr->n_gpus <= 64 && pr->n_edges >= 0, TS_ERR_INVALID_ARG,
             "%s: bad sizes (kernels %d, gpus %d, edges %d)", who, pr->n_kernels, pr->n_gpus, pr->n_edges);
  TS_REQUIRE(pr->t != nullptr && (pr->n_edges == 0 || pr->edges != nullptr) && (pr->n_gpus == 1 || (pr->bw && pr->lat)),
             TS_ERR_INVALID_ARG, "%s: null table", who);
  TS_REQUIRE(objective == TS_PLAN_THROUGHPUT || objective == TS_PLAN_LATENCY, TS_ERR_INVALID_ARG,
             "%s: unknown objective %d", who, objective);
  TS_REQUIRE(rel_gap >= 0.0 && rel_gap < 1.0, TS_ERR_INVALID_ARG, "%s: rel_gap %g outside [0, 1)", who, rel_gap);
  Problem p;
  p.K = pr->n_kernels;
  p.G = pr->n_gpus;
  p.t = pr->t;
  p.bw = pr->bw;
  p.lat = pr->lat;
  p.in.resize(p.K);
  for (int e = 0; e < pr->n_edges; ++e) {
    const ts_ddg_edge& ed = pr->edges[e];
    if (ed.cross_iteration) continue;                      // replicated buffers: no cost in the objectives
    TS_REQUIRE(ed.src >= 0 && ed.src < ed.dst && ed.dst < p.K, TS_ERR_INVALID_ARG,
               "%s: edge %d (%d -> %d) does not follow execution order", who, e, ed.src, ed.dst);
    p.in[ed.dst].push_back({ed.src, (double)ed.bytes});
  }
  for (int i = 0; i < p.K * p.G; ++i)
    TS_REQUIRE(pr->t[i] >= 0.0 && std::isfinite(pr->t[i]), TS_ERR_INVALID_ARG, "%s: negative or non-finite latency", who);

  BnB s{p, objective, node_limit > 0 ? node_limit : (int64_t)50'000'000};
  s.T.assign(p.G, 0.0);
  s.M.assign(p.G, 0.0);
  s.place.assign(p.K, 0);
  s.rem_min.assign(p.K + 1, 0.0);
  for (int k = p.K - 1; k >= 0; --k) {
    double mn = p.t[k * p.G];
    for (int g = 1; g < p.G; ++g) mn = std::min(mn, p.t[k * p.G + g]);
    s.rem_min[k] = s.rem_min[k + 1] + mn;
  }
  if (p.G == 2) {
    s.rem0.assign(p.K + 1, 0.0);
    for (int k = p.K - 1; k >= 0; --k) s.rem0[k] = s.rem0[k + 1] + p.t[k * 2];
    s.by_ratio.resize(p.K);
    for (int k = 0; k < p.K; ++k) s.by_ratio[k] = k;
    auto ratio = [&](int x) {
      return p.t[x * 2] > 0.0 ? p.t[x * 2 + 1] / p.t[x * 2] : std::numeric_limits<double>::infinity();
    };
    std::stable_sort(s.by_ratio.begin(), s.by_ratio.end(), [&](int x, int y) { return ratio(x) < ratio(y); });
    if (objective == TS_PLAN_THROUGHPUT && placement != nullptr) s.build_fractional_tables();
  }
  const double root_bound = s.bound(0);                    // nothing placed yet: a bound of the optimum itself
  if (placement == nullptr) {                              // bound only
    *lower_bound = root_bound;
    return TS_OK;
  }

  std::vector<int32_t> best_place;
  double best = 0.0;
  int st = 2;
  if (!(objective == TS_PLAN_LATENCY && plan_latency_dp(p, best_place, best))) {
    s.rel_gap = rel_gap;
    s.root_lb = root_bound;
    // incumbent: the best single GPU (always feasible, no communication)
    for (int g = 0; g < p.G; ++g) {
      double v = 0.0;
      for (int k = 0; k < p.K; ++k) v += p.t[k * p.G + g];
      if (v < s.best) { s.best = v; s.best_place.assign(p.K, g); }
    }
    if (p.G > 1 && p.K <= 4096) {
      std::vector<int32_t> seed;
      std::vector<double> T, M;
      contiguous_seed(p, seed);
      evaluate(p, seed.data(), T, M);
      s.T = T; s.M = M;
      const double v = s.bound(p.K);                     // with every kernel placed the bound is the objective
      if (v < s.best) { s.best = v; s.best_place = seed; }
      s.T.assign(p.G, 0.0);
      s.M.assign(p.G, 0.0);
    }
    // two GPUs, throughput: balance the incumbent by whole classes of equal kernels before and after the search
    const bool polish = objective == TS_PLAN_THROUGHPUT && p.G == 2;
    Polish fine(p);
    auto polish_rounds = [&]() {
      for (int round = 0; polish && round < 6 && !s.close_enough(); ++round)
        if (!fine.run(s.best_place, s.best)) break;
    };
    polish_rounds();
    bool complete = false;                               // the branch and bound ran to its end
    if (!s.close_enough()) {
      s.dfs(0);
      complete = !s.exhausted;
      if (!complete && !s.within_gap) polish_rounds();
    }
    best_place = s.best_place;
    st = complete ? 2 : (s.close_enough() ? 1 : 0);
  }
  std::vector<double> T, M;
  evaluate(p, best_place.data(), T, M);
  double v = 0.0;
  if (objective == TS_PLAN_THROUGHPUT) {
    for (int g = 0; g < p.G; ++g) v = std::max(v, std::max(T[g], M[g]));
  } else {
    for (int g = 0; g < p.G; ++g) v += T[g];
    for (int g = 0; g < p.G; ++g) v += M[g];
  }
  std::copy(best_place.begin(), best_place.end(), placement);
  *value = v;
  if (T_g) std::copy(T.begin(), T.end(), T_g);
  if (M_g) std::copy(M.begin(), M.end(), M_g);
  if (status) *status = st;
  if (lower_bound) *lower_bound = st == 2 ? v : std::min(v, root_bound);
  return TS_OK;
}

int ts_plan_policy(const ts_plan_problem* pr, int objective, int64_t node_limit, int32_t* placement, double* value,
                   double* T_g, double* M_g, int* proved_optimal) {
  TS_REQUIRE(placement != nullptr && value != nullptr, TS_ERR_INVALID_ARG, "ts_plan_policy: null argument");
  int st = 0;
  int rc = plan_impl(pr, objective, node_limit, 0.0, placement, value, T_g, M_g, &st, nullptr, "ts_plan_policy");
  if (rc == TS_OK && proved_optimal) *proved_optimal = st == 2 ? 1 : 0;
  return rc;
}

int ts_plan_policy_bounded(const ts_plan_problem* pr, int objective, int64_t node_limit, double rel_gap,
                           int32_t* placement, double* value, double* T_g, double* M_g, double* lower_bound,
                           int* status) {
  TS_REQUIRE(placement != nullptr && value != nullptr, TS_ERR_INVALID_ARG, "ts_plan_policy_bounded: null argument");
  return plan_impl(pr, objective, node_limit, rel_gap, placement, value, T_g, M_g, status, lower_bound,
                   "ts_plan_policy_bounded");
}

int ts_plan_lower_bound(const ts_plan_problem* pr, int objective, double* lower_bound) {
  TS_REQUIRE(lower_bound != nullptr, TS_ERR_INVALID_ARG, "ts_plan_lower_bound: null argument");
  return plan_impl(pr, objective, 0, 0.0, nullptr, nullptr, nullptr, nullptr, nullptr, lower_bound, "ts_plan_lower_bound");
}

}  // extern "C"
