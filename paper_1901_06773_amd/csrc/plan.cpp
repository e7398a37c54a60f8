// Planner: cost model (Eq. 2, Eq. 5), memory model (Eq. 4), t_ready (Algorithm 1), the
// no-stall test (Eq. 6) and the swap / pin decision (body of Algorithm 2).
#include "plan.h"

#include <algorithm>
#include <chrono>
#include <cstdio>

namespace acc {

// ------------------------------------------------------------------------- cost model
double CostModel::step_time(const Graph& g, int step, int k) const {
  if (!fixed.empty() && step < (int)fixed.size()) return fixed[step];
  if (!ks.empty()) {
    // measured times; between two measured minibatches interpolate linearly in k, beyond the
    // largest one scale in proportion (throughput saturated, Sec. 3.3.1), below the smallest
    // scale down but never under the launch cost
    const int n = (int)ks.size();
    if (k >= ks[n - 1]) return table[n - 1][step] * ((double)k / ks[n - 1]);
    if (k <= ks[0]) return std::max(launch_s, table[0][step] * ((double)k / ks[0]));
    int i = 1;
    while (ks[i] < k) ++i;
    const double f = (double)(k - ks[i - 1]) / (ks[i] - ks[i - 1]);
    return table[i - 1][step] * (1.0 - f) + table[i][step] * f;
  }
  const Step& s = g.steps[step];
  return launch_s + s.flops_per_image * k / flops_per_s +
         (s.bytes_per_image * k + s.bytes_fixed) / bytes_per_s;
}

// ------------------------------------------------------------------------------ arena
namespace {

struct Seg {
  size_t off, size;
  int tag_step, tag_d2h;   // what must have finished before the bytes may be written again
};

class Arena {
 public:
  explicit Arena(size_t cap, bool best_fit = false) : best_fit_(best_fit) { free_.push_back({0, cap, -1, -1}); }

  // First fit; blocks whose offload has a sequence number above `ready_d2h` (still being
  // copied out) are used only if nothing else fits.
  bool alloc(size_t need, bool top, int ready_d2h, size_t* off, int* dstep, int* dd2h) {
    if (try_alloc(need, top, ready_d2h, off, dstep, dd2h)) return true;
    return try_alloc(need, top, 1 << 30, off, dstep, dd2h);
  }

  // First fit over runs of adjacent free segments; bottom-up, or top-down for long-lived
  // objects so that they do not fragment the space the short-lived ones cycle through.
  // Segments with tag_d2h > limit do not count as free.
  bool try_alloc(size_t need, bool top, int limit, size_t* off, int* dstep, int* dd2h) {
    const int n = (int)free_.size();
    auto usable = [&](int q) { return free_[q].tag_d2h <= limit; };
    *dstep = -1;
    *dd2h = -1;
    if (best_fit_ && need > 0) {
      // maximal runs of adjacent usable segments; the smallest one that holds the block wins
      // (bottom-up blocks sit at its low end, top-down blocks at its high end)
      int bi = -1, bj = -1;
      size_t bsize = 0;
      for (int i = 0; i < n;) {
        if (!usable(i)) { ++i; continue; }
        int j = i;
        size_t total = free_[i].size;
        while (j + 1 < n && usable(j + 1) && free_[j + 1].off == free_[j].off + free_[j].size) total += free_[++j].size;
        if (total >= need && (bi < 0 || total < bsize)) { bi = i; bj = j; bsize = total; }
        i = j + 1;
      }
      if (bi < 0) return false;
      return take_from_run(bi, bj, need, top, off, dstep, dd2h);
    }
    if (!top) {
      int i = 0;
      while (i < n) {
        if (!usable(i)) { ++i; continue; }
        size_t total = 0;
        int j = i;
        for (;;) {
          total += free_[j].size;
          if (total >= need) break;
          if (j + 1 < n && free_[j + 1].off == free_[j].off + free_[j].size && usable(j + 1)) ++j;
          else { total = 0; break; }
        }
        if (total >= need && need > 0) {
          *off = free_[i].off;
          for (int q = i; q <= j; ++q) {
            *dstep = std::max(*dstep, free_[q].tag_step);
            *dd2h = std::max(*dd2h, free_[q].tag_d2h);
          }
          const size_t rest = total - need;
          if (rest) {
            free_[j].off = free_[j].off + free_[j].size - rest;
            free_[j].size = rest;
            free_.erase(free_.begin() + i, free_.begin() + j);
          } else {
            free_.erase(free_.begin() + i, free_.begin() + j + 1);
          }
          return true;
        }
        i = j + 1;
      }
      return false;
    }
    int i = n - 1;
    while (i >= 0) {
      if (!usable(i)) { --i; continue; }
      size_t total = 0;
      int j = i;
      for (;;) {
        total += free_[j].size;
        if (total >= need) break;
        if (j - 1 >= 0 && free_[j - 1].off + free_[j - 1].size == free_[j].off && usable(j - 1)) --j;
        else { total = 0; break; }
      }
      if (total >= need && need > 0) {
        *off = free_[i].off + free_[i].size - need;
        for (int q = j; q <= i; ++q) {
          *dstep = std::max(*dstep, free_[q].tag_step);
          *dd2h = std::max(*dd2h, free_[q].tag_d2h);
        }
        const size_t rest = total - need;
        if (rest) {
          free_[j].size = rest;
          free_.erase(free_.begin() + j + 1, free_.begin() + i + 1);
        } else {
          free_.erase(free_.begin() + j, free_.begin() + i + 1);
        }
        return true;
      }
      i = j - 1;
    }
    return false;
  }

  // carves `need` bytes out of the run of adjacent segments [i, j]: from its low end, or from its
  // high end for top-down blocks; segments that are used up disappear, one may shrink
  bool take_from_run(int i, int j, size_t need, bool top, size_t* off, int* dstep, int* dd2h) {
    size_t left = need;
    if (!top) {
      *off = free_[i].off;
      int q = i;
      while (left > 0) {
        *dstep = std::max(*dstep, free_[q].tag_step);
        *dd2h = std::max(*dd2h, free_[q].tag_d2h);
        if (free_[q].size <= left) { left -= free_[q].size; ++q; }
        else { free_[q].off += left; free_[q].size -= left; left = 0; }
      }
      free_.erase(free_.begin() + i, free_.begin() + q);
    } else {
      *off = free_[j].off + free_[j].size - need;
      int q = j;
      while (left > 0) {
        *dstep = std::max(*dstep, free_[q].tag_step);
        *dd2h = std::max(*dd2h, free_[q].tag_d2h);
        if (free_[q].size <= left) { left -= free_[q].size; --q; }
        else { free_[q].size -= left; left = 0; }
      }
      free_.erase(free_.begin() + q + 1, free_.begin() + j + 1);   // the segments used up entirely
    }
    return true;
  }

  void release(size_t off, size_t size, int tag_step, int tag_d2h) {
    Seg s{off, size, tag_step, tag_d2h};
    auto it = std::lower_bound(free_.begin(), free_.end(), s,
                               [](const Seg& a, const Seg& b) { return a.off < b.off; });
    it = free_.insert(it, s);
    // merge with neighbours that carry the same tags
    const int i = (int)(it - free_.begin());
    if (i + 1 < (int)free_.size() && free_[i].off + free_[i].size == free_[i + 1].off &&
        free_[i].tag_step == free_[i + 1].tag_step && free_[i].tag_d2h == free_[i + 1].tag_d2h) {
      free_[i].size += free_[i + 1].size;
      free_.erase(free_.begin() + i + 1);
    }
    if (i > 0 && free_[i - 1].off + free_[i - 1].size == free_[i].off &&
        free_[i - 1].tag_step == free_[i].tag_step && free_[i - 1].tag_d2h == free_[i].tag_d2h) {
      free_[i - 1].size += free_[i].size;
      free_.erase(free_.begin() + i);
    }
  }

 private:
  std::vector<Seg> free_;
  bool best_fit_ = false;
};

enum TState { TS_NONE = 0, TS_FWD, TS_OFFLOADED, TS_RESIDENT, TS_DEAD };

}  // namespace

// ------------------------------------------------------------------------- build_plan
static bool build_plan_once(const Graph& g, int k, size_t budget, const std::vector<uint8_t>& swap_of_tensor,
                            const PlanOptions& opt, Plan* out, std::string* why) {
  Plan& P = *out;
  P = Plan();
  P.k = k;
  P.budget = budget;
  const int nt = (int)g.tensors.size(), ns = (int)g.steps.size();
  if (k <= 0) { *why = "minibatch must be positive"; return false; }
  P.swapped.assign(nt, 0);
  P.off1.assign(nt, 0); P.off2.assign(nt, 0); P.host_off.assign(nt, 0); P.tbytes.assign(nt, 0);
  for (int t = 0; t < nt; ++t) {
    P.tbytes[t] = g.bytes(t, k);
    if (t < (int)swap_of_tensor.size() && swap_of_tensor[t] && g.tensors[t].is_map) P.swapped[t] = 1;
  }
  const size_t stat = g.static_bytes();
  if (!opt.unlimited && budget < stat + 256) { *why = "budget below the resident parameters and gradients"; return false; }
  const size_t cap = opt.unlimited ? ((size_t)1 << 56) : ((budget - stat) & ~(size_t)255);
  Arena arena(cap, opt.best_fit);

  std::vector<int> st(nt, TS_NONE), d2h_of(nt, -1), h2d_of(nt, -1);
  std::vector<size_t> cur_off(nt, 0);
  std::vector<int> step_wait_d2h(ns, -1);
  std::vector<char> step_record(ns, 0);
  std::vector<std::vector<int>> free_after(ns), offload_after(ns);
  for (int t = 0; t < nt; ++t) {
    const Tensor& T = g.tensors[t];
    if (P.swapped[t]) offload_after[T.last_fwd].push_back(t);
    free_after[T.last].push_back(t);
  }
  // the model's clock (stalls ignored, so it runs early and errs towards "still copying")
  double clk = 0.0, link_out = 0.0;
  std::vector<double> d2h_done;                 // per offload sequence number
  auto ready_d2h = [&]() {
    if (!opt.clock) return 1 << 30;
    int r = -1;
    while (r + 1 < (int)d2h_done.size() && d2h_done[r + 1] <= clk) ++r;
    return r;
  };
  size_t live = 0;
  auto take = [&](int t, bool top, int* dstep, int* dd2h) {
    size_t off = 0;
    if (!arena.alloc(P.tbytes[t], top, ready_d2h(), &off, dstep, dd2h)) return false;
    cur_off[t] = off;
    live += P.tbytes[t];
    if (live > P.dyn_peak) P.dyn_peak = live;
    if (!top && off + P.tbytes[t] > P.dyn_extent) P.dyn_extent = off + P.tbytes[t];
    if (off + P.tbytes[t] > P.dyn_top) P.dyn_top = off + P.tbytes[t];
    return true;
  };
  auto long_lived = [&](int t) { return g.tensors[t].is_map && !P.swapped[t]; };

  // the input batch is the first layer's prefetch (Algorithm 1, j == 1)
  for (int t : {g.t_stage, g.t_labels}) {
    int ds, dd;
    if (!take(t, long_lived(t), &ds, &dd)) { *why = "input batch does not fit"; return false; }
    P.off1[t] = cur_off[t];
    st[t] = P.swapped[t] ? TS_FWD : TS_RESIDENT;
    Instr in;
    in.op = I_LOAD_INPUT; in.arg = t; in.seq = P.n_h2d++;
    h2d_of[t] = in.seq;
    P.instrs.push_back(in);
  }

  // running ahead of the compute stream only pays while some map still has to come back
  int to_prefetch = 0;
  for (int t = 0; t < nt; ++t) to_prefetch += P.swapped[t];

  // allocations (and prefetches) of one step, in order; forced = the step is about to run
  auto alloc_step = [&](int j, bool forced) -> bool {
    const Step& s = g.steps[j];
    Arena snap = arena;
    const size_t live0 = live, peak0 = P.dyn_peak, ext0 = P.dyn_extent, top0 = P.dyn_top;
    const size_t n_instr0 = P.instrs.size();
    const int n_h2d0 = P.n_h2d;
    std::vector<std::pair<int, int>> undo;   // tensor, previous state
    auto rollback = [&]() {
      arena = snap; live = live0; P.dyn_peak = peak0; P.dyn_extent = ext0; P.dyn_top = top0;
      P.instrs.resize(n_instr0); P.n_h2d = n_h2d0;
      for (auto& u : undo) {
        st[u.first] = u.second;
        if (u.second == TS_OFFLOADED) { h2d_of[u.first] = -1; ++to_prefetch; }
      }
      step_wait_d2h[j] = -1;
    };
    for (int t : s.reads) {
      if (st[t] == TS_FWD && P.swapped[t] && g.tensors[t].last_fwd < j && !forced) {
        // still waiting to be offloaded: its backward copy cannot be placed yet
        rollback();
        return false;
      }
      if (st[t] == TS_OFFLOADED) {
        int ds, dd;
        if (!take(t, false, &ds, &dd)) { rollback(); return false; }
        undo.push_back({t, TS_OFFLOADED});
        st[t] = TS_RESIDENT;
        P.off2[t] = cur_off[t];
        --to_prefetch;
        Instr pf;
        pf.op = I_PREFETCH; pf.arg = t; pf.seq = P.n_h2d++;
        pf.wait_step = ds;
        pf.wait_d2h = std::max(dd, d2h_of[t]);
        h2d_of[t] = pf.seq;
        if (ds >= 0) step_record[ds] = 1;
        P.instrs.push_back(pf);
      } else if (st[t] == TS_NONE || st[t] == TS_DEAD) {
        rollback();
        *why = "internal: step reads a tensor that is not alive";
        return false;
      }
    }
    for (int t : s.writes) {
      if (st[t] != TS_NONE) continue;
      int ds, dd;
      if (!take(t, long_lived(t), &ds, &dd)) { rollback(); return false; }
      undo.push_back({t, TS_NONE});
      st[t] = P.swapped[t] ? TS_FWD : TS_RESIDENT;
      P.off1[t] = cur_off[t];
      step_wait_d2h[j] = std::max(step_wait_d2h[j], dd);
    }
    return true;
  };

  // eager prefetch: swapped maps in the order of their first use in backward
  std::vector<int> eager_order;
  size_t next_eager = 0;
  if (opt.eager_headroom) {
    for (int t = 0; t < nt; ++t)
      if (P.swapped[t]) eager_order.push_back(t);
    std::stable_sort(eager_order.begin(), eager_order.end(),
                     [&](int a, int b) { return g.tensors[a].first_bwd < g.tensors[b].first_bwd; });
  }
  auto eager_prefetch = [&]() {
    while (next_eager < eager_order.size()) {
      const int t = eager_order[next_eager];
      if (st[t] == TS_RESIDENT || st[t] == TS_DEAD) { ++next_eager; continue; }   // came back with its step
      if (st[t] != TS_OFFLOADED) break;
      if (live + P.tbytes[t] + opt.eager_headroom > cap) break;
      int ds, dd;
      if (!take(t, true, &ds, &dd)) break;
      st[t] = TS_RESIDENT;
      P.off2[t] = cur_off[t];
      --to_prefetch;
      Instr pf;
      pf.op = I_PREFETCH; pf.arg = t; pf.seq = P.n_h2d++;
      pf.wait_step = ds;
      pf.wait_d2h = std::max(dd, d2h_of[t]);
      h2d_of[t] = pf.seq;
      if (ds >= 0) step_record[ds] = 1;
      P.instrs.push_back(pf);
      ++next_eager;
    }
  };

  int ahead = 0;
  int seen_c_d2h = -1, seen_c_h2d = -1;

  for (int j = 0; j < ns; ++j) {
    while (ahead <= j) {
      *why = "";
      if (!alloc_step(ahead, true)) {
        if (why->empty()) {
          char buf[160];
          snprintf(buf, sizeof buf, "step %d (%s) does not fit the budget at minibatch %d", ahead,
                   step_kind_name(g.steps[ahead].kind), k);
          *why = buf;
        }
        return false;
      }
      ++ahead;
    }
    if (opt.lookahead && !opt.eager_headroom)
      while (ahead < ns && ahead >= g.n_fwd && to_prefetch > 0) {
        if (!alloc_step(ahead, false)) break;
        ++ahead;
      }
    Instr c;
    c.op = I_COMPUTE; c.arg = j;
    if (step_wait_d2h[j] > seen_c_d2h) { c.wait_d2h = step_wait_d2h[j]; seen_c_d2h = c.wait_d2h; }
    int need_h2d = -1;
    for (int t : g.steps[j].reads) need_h2d = std::max(need_h2d, h2d_of[t]);
    if (need_h2d > seen_c_h2d) { c.wait_h2d = need_h2d; seen_c_h2d = need_h2d; }
    P.instrs.push_back(c);
    if (opt.clock) clk += opt.clock->step_time(g, j, k);

    for (int t : offload_after[j]) {
      Instr o;
      o.op = I_OFFLOAD; o.arg = t; o.wait_step = j; o.seq = P.n_d2h++;
      step_record[j] = 1;
      d2h_of[t] = o.seq;
      P.host_off[t] = P.host_bytes;
      P.host_bytes += P.tbytes[t];
      P.bytes_swapped += P.tbytes[t];
      ++P.n_swapped;
      P.instrs.push_back(o);
      if (opt.clock) {
        link_out = std::max(link_out, clk) + opt.clock->d2h_time(P.tbytes[t]);
        d2h_done.push_back(link_out);
      }
      arena.release(cur_off[t], P.tbytes[t], -1, o.seq);
      live -= P.tbytes[t];
      st[t] = TS_OFFLOADED;
      h2d_of[t] = -1;
    }
    for (int t : free_after[j]) {
      if (st[t] == TS_RESIDENT || st[t] == TS_FWD) {
        arena.release(cur_off[t], P.tbytes[t], j, -1);
        live -= P.tbytes[t];
        st[t] = TS_DEAD;
      }
    }
    if (opt.eager_headroom && j + 1 >= g.n_fwd && to_prefetch > 0) eager_prefetch();
  }
  *why = "";
  // the swap-in stream waits in order too: drop waits it has already passed
  int seen_i_step = -1, seen_i_d2h = -1;
  for (Instr& in : P.instrs) {
    if (in.op == I_COMPUTE) in.record = step_record[in.arg] != 0;
    if (in.op == I_PREFETCH) {
      if (in.wait_step <= seen_i_step) in.wait_step = -1; else seen_i_step = in.wait_step;
      if (in.wait_d2h <= seen_i_d2h) in.wait_d2h = -1; else seen_i_d2h = in.wait_d2h;
    }
  }
  P.valid = true;
  return true;
}

bool build_plan(const Graph& g, int k, size_t budget, const std::vector<uint8_t>& swap_of_tensor,
                const PlanOptions& opt, Plan* out, std::string* why) {
  if (build_plan_once(g, k, budget, swap_of_tensor, opt, out, why)) return true;
  if (!opt.lookahead) return false;
  // Running ahead changes where blocks land; if that fragments the pool so far that a
  // step no longer fits, fall back to just-in-time allocation, which needs the least.
  PlanOptions jit = opt;
  jit.lookahead = false;
  std::string why2;
  if (build_plan_once(g, k, budget, swap_of_tensor, jit, out, &why2)) { *why = ""; return true; }
  // ... and if first fit still cannot place a step, best fit, which fragments less
  jit.best_fit = true;
  if (build_plan_once(g, k, budget, swap_of_tensor, jit, out, &why2)) { *why = ""; return true; }
  return false;
}

// --------------------------------------------------------------------------- simulate
void simulate(const Graph& g, const CostModel& cm, Plan* plan) {
  Plan& P = *plan;
  const int ns = (int)g.steps.size();
  P.t_cost.assign(ns, 0); P.t_ready.assign(ns, 0); P.t_start.assign(ns, 0); P.t_end.assign(ns, 0);
  std::vector<double> d2h_t(P.n_d2h, 0), h2d_t(P.n_h2d, 0);
  double t_c = 0, t_o = 0, t_i = 0, stall = 0, comp = 0;
  // waits already passed still bound a stream from below: keep the running maximum
  double c_floor = 0, i_floor = 0;
  P.i_start.assign(P.instrs.size(), 0); P.i_end.assign(P.instrs.size(), 0);
  size_t ii = 0;
  for (const Instr& in : P.instrs) {
    double& i_start = P.i_start[ii];
    double& i_end = P.i_end[ii];
    ++ii;
    switch (in.op) {
      case I_LOAD_INPUT: {
        const double end = t_i + cm.h2d_time(P.tbytes[in.arg]);
        i_start = t_i; i_end = end;
        h2d_t[in.seq] = end;
        t_i = end;
        break;
      }
      case I_COMPUTE: {
        const int j = in.arg;
        if (in.wait_d2h >= 0) c_floor = std::max(c_floor, d2h_t[in.wait_d2h]);
        if (in.wait_h2d >= 0) c_floor = std::max(c_floor, h2d_t[in.wait_h2d]);
        const double cost = cm.step_time(g, j, P.k);
        P.t_cost[j] = cost;
        P.t_ready[j] = c_floor;
        const double start = std::max(t_c, c_floor);
        stall += start - t_c;
        P.t_start[j] = start;
        P.t_end[j] = start + cost;
        i_start = start; i_end = start + cost;
        t_c = start + cost;
        comp += cost;
        break;
      }
      case I_OFFLOAD: {
        const double start = std::max(t_o, P.t_end[in.wait_step]);
        const double end = start + cm.d2h_time(P.tbytes[in.arg]);
        i_start = start; i_end = end;
        d2h_t[in.seq] = end;
        t_o = end;
        break;
      }
      case I_PREFETCH: {
        if (in.wait_step >= 0) i_floor = std::max(i_floor, P.t_end[in.wait_step]);
        if (in.wait_d2h >= 0) i_floor = std::max(i_floor, d2h_t[in.wait_d2h]);
        const double start = std::max(t_i, i_floor);
        const double end = start + cm.h2d_time(P.tbytes[in.arg]);
        i_start = start; i_end = end;
        h2d_t[in.seq] = end;
        t_i = end;
        break;
      }
    }
  }
  P.t_compute = comp;
  P.t_stall = stall;
  P.t_iter = std::max(t_c, std::max(t_o, t_i));
}

size_t live_peak(const Graph& g, int k, const std::vector<uint8_t>& swap_of_tensor) {
  Plan p;
  std::string why;
  PlanOptions o;
  o.lookahead = false;
  o.unlimited = true;
  if (!build_plan(g, k, 0, swap_of_tensor, o, &p, &why)) return 0;
  return p.dyn_peak;
}

// -------------------------------------------------------------------------- make_plan
int make_plan(const Graph& g, const CostModel& cm, int k, size_t budget, int mode, Plan* out,
              std::string* why) {
  const int nt = (int)g.tensors.size();
  std::vector<uint8_t> none(nt, 0), all(nt, 0);
  for (int t : g.maps) all[t] = 1;
  PlanOptions opt;
  if (budget < g.static_bytes() + 256) {
    *why = "budget below the resident parameters and gradients";
    return ACC_EPOOL;
  }
  if (mode == ACC_PLAN_NONE) {
    if (!build_plan(g, k, budget, none, opt, out, why)) return ACC_EPOOL;
    simulate(g, cm, out);
    out->mode = mode;
    return ACC_OK;
  }
  // A swap set is laid out three times: with plain first fit, with first fit that passes over
  // blocks still being copied out (by the model's clock), and with eager prefetch on top of
  // that; the layout with the shortest predicted iteration is kept.
  const size_t headroom = live_peak(g, k, all);   // working set of the steps: peak with every map away
  auto build_sim = [&](const std::vector<uint8_t>& sw, Plan* p, std::string* w) -> bool {
    Plan pa, pb;
    std::string wa, wb;
    const bool oka = build_plan(g, k, budget, sw, opt, &pa, &wa);
    if (oka) simulate(g, cm, &pa);
    PlanOptions timed = opt;
    timed.clock = &cm;
    const bool okb = build_plan(g, k, budget, sw, timed, &pb, &wb);
    if (okb) simulate(g, cm, &pb);
    // third layout: maps come back as early as the pool has room beside the working set
    Plan pc;
    std::string wc;
    PlanOptions eager = timed;
    eager.eager_headroom = headroom;
    const bool okc = headroom > 0 && build_plan(g, k, budget, sw, eager, &pc, &wc);
    if (okc) simulate(g, cm, &pc);
    if (!oka && !okb && !okc) { *w = wa; return false; }
    Plan* bestp = nullptr;
    for (Plan* q : {oka ? &pa : nullptr, okb ? &pb : nullptr, okc ? &pc : nullptr})
      if (q && (!bestp || q->t_iter < bestp->t_iter)) bestp = q;
    *p = std::move(*bestp);
    return true;
  };
  // Last pass over the chosen swap set: eager prefetch that keeps less than the whole working
  // set free.  The working-set peak lies at the large early layers, which backward reaches
  // last, so at the start of backward less room is enough and the link need not wait for it;
  // a layout in which some step then finds no room is dropped (build_plan fails), the others
  // are simulated and the fastest is kept.
  auto refine_layout = [&](const std::vector<uint8_t>& sw, Plan* best) {
    if (headroom == 0 || best->n_swapped == 0) return;
    for (double f : {0.75, 0.5, 0.25, 0.125}) {
      PlanOptions eager = opt;
      eager.clock = &cm;
      eager.eager_headroom = std::max<size_t>(256, (size_t)(headroom * f));
      Plan p;
      std::string w;
      if (!build_plan(g, k, budget, sw, eager, &p, &w)) continue;
      simulate(g, cm, &p);
      if (p.t_iter < best->t_iter * (1.0 - 1e-6)) *best = std::move(p);
    }
  };
  if (mode == ACC_PLAN_NAIVE_ALL) {
    if (!build_sim(all, out, why)) return ACC_EUNTRAINABLE;
    refine_layout(all, out);
    out->mode = mode;
    return ACC_OK;
  }
  if (mode != ACC_PLAN_DYNAMIC) { *why = "unknown planner mode"; return ACC_EINVAL; }

  // If nothing has to leave the GPU, nothing does (the swap-none plan has no stall at all).
  if (build_plan(g, k, budget, none, opt, out, why)) {
    simulate(g, cm, out);
    out->mode = mode;
    return ACC_OK;
  }
  // Trainability: the layer-wise peak with every map swapped must fit (k <= k_max).
  Plan best;
  if (!build_sim(all, &best, why)) return ACC_EUNTRAINABLE;
  // Pin maps back into the memory the active area leaves free, starting with the maps
  // produced last (needed first in backward: the ones whose prefetch cannot hide), and keep
  // a pin whenever the predicted iteration does not get slower.
  std::vector<uint8_t> cur = all;
  for (int pass = 0; pass < 4; ++pass) {
    bool changed = false;
    for (int i = (int)g.maps.size() - 1; i >= 0; --i) {
      const int t = g.maps[i];
      if (!cur[t]) continue;
      cur[t] = 0;
      Plan trial;
      std::string w2;
      if (build_sim(cur, &trial, &w2)) {
        if (trial.t_iter <= best.t_iter * (1.0 + 1e-9)) {
          best = std::move(trial);
          changed = true;
          continue;
        }
      }
      cur[t] = 1;
    }
    if (!changed) break;
  }
  // Local refinement: move a swap to a neighbouring map (in producer order) when that
  // shortens the predicted iteration; which of two adjacent maps leaves the GPU decides
  // how well its copies hide behind the steps in between.
  const int nm = (int)g.maps.size();
  for (int pass = 0; pass < 2; ++pass) {
    bool changed = false;
    for (int i = 0; i < nm; ++i) {
      if (!cur[g.maps[i]]) continue;
      for (int d = -2; d <= 2; ++d) {
        const int j = i + d;
        if (d == 0 || j < 0 || j >= nm || cur[g.maps[j]] || !cur[g.maps[i]]) continue;
        cur[g.maps[i]] = 0;
        cur[g.maps[j]] = 1;
        Plan trial;
        std::string w2;
        bool better = false;
        if (build_sim(cur, &trial, &w2)) better = trial.t_iter < best.t_iter * (1.0 - 1e-6);
        if (better) {
          best = std::move(trial);
          changed = true;
        } else {
          cur[g.maps[i]] = 1;
          cur[g.maps[j]] = 0;
        }
      }
    }
    if (!changed) break;
  }
  refine_layout(cur, &best);
  *out = std::move(best);
  out->mode = mode;
  *why = "";
  return ACC_OK;
}

}  // namespace acc
