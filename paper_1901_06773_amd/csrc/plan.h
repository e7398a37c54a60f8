// Performance model, Algorithm 1 and the body of Algorithm 2 of the paper, on the host.
//
// A plan is an instruction list for three streams (compute, swap-out, swap-in; Sec. 5)
// with pool offsets fixed ahead of time.  Memory reuse is ordered by events that are part
// of the plan: a block may be written again only after the last use of its previous
// occupant (a kernel or an offload copy) has finished.  The same list is interpreted twice:
// by simulate() with the cost model, giving t_ready (Algorithm 1), the no-stall test
// (Eq. 6) and the predicted iteration time (Eq. 2 plus stalls), and by the executor with
// real streams and events.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "graph.h"

namespace acc {

struct CostModel {
  // synthetic model (used until calibrated)
  double flops_per_s = 60e12, bytes_per_s = 3e12, launch_s = 6e-6;
  double d2h_bps = 50e9, h2d_bps = 50e9, copy_latency_s = 12e-6;
  // measured table: seconds per step at minibatch ks[i] (ascending)
  std::vector<int> ks;
  std::vector<std::vector<double>> table;
  // explicit per-step override (tests of Algorithm 1)
  std::vector<double> fixed;

  double step_time(const Graph& g, int step, int k) const;
  double d2h_time(size_t bytes) const { return copy_latency_s + (double)bytes / d2h_bps; }
  double h2d_time(size_t bytes) const { return copy_latency_s + (double)bytes / h2d_bps; }
};

enum InstrOp { I_LOAD_INPUT = 0, I_COMPUTE = 1, I_OFFLOAD = 2, I_PREFETCH = 3 };

struct Instr {
  int op = 0;
  int arg = -1;          // tensor id, or step index for I_COMPUTE
  int wait_step = -1;    // wait for the event recorded after this compute step
  int wait_d2h = -1;     // wait for the offload with this sequence number
  int wait_h2d = -1;     // wait for the prefetch / input load with this sequence number
  int seq = -1;          // own sequence number among offloads resp. prefetches+loads
  bool record = false;   // I_COMPUTE: another stream waits for this step
};

struct Plan {
  int k = 0;
  size_t budget = 0;           // whole budget, static part included
  int mode = 0;
  bool valid = false;
  std::vector<uint8_t> swapped;            // per tensor
  std::vector<size_t> off1, off2, host_off;  // per tensor: first allocation, after prefetch, host slot
  std::vector<size_t> tbytes;              // per tensor size at k
  std::vector<Instr> instrs;
  int n_d2h = 0, n_h2d = 0;
  size_t dyn_peak = 0;                     // high-water sum of live dynamic bytes
  size_t dyn_extent = 0;                   // highest pool offset + size used by bottom-up blocks
  size_t dyn_top = 0;                      // highest pool offset + size of any block (top-down ones included)
  size_t host_bytes = 0;
  size_t bytes_swapped = 0;
  int n_swapped = 0;
  // simulation results
  std::vector<double> t_cost, t_ready, t_start, t_end;
  std::vector<double> i_start, i_end;      // per instruction, on its own stream
  double t_iter = 0, t_stall = 0, t_compute = 0;
};

struct PlanOptions {
  bool lookahead = true;       // run allocations / prefetches ahead of the compute stream
  bool unlimited = false;      // ignore the budget (only to measure peaks)
  // With a cost model: a block that an offload is still copying out (by the model's clock)
  // is passed over while any other free block fits, so that an allocation does not wait for
  // a copy when untouched memory is at hand.  Without: plain first fit.
  const CostModel* clock = nullptr;
  // > 0: in backward, bring swapped maps back as soon as the pool has room for the map plus
  // this many bytes (kept free for the working set of the steps in between), in the order
  // of their first use, instead of running the allocations of whole steps ahead.
  size_t eager_headroom = 0;
  // Among the free runs that are large enough take the smallest instead of the first (less
  // fragmentation; tried when first fit cannot place a step).
  bool best_fit = false;
};

// Builds instruction list and placement for a fixed swap set.  Returns false (and why)
// when some allocation does not fit the budget.
bool build_plan(const Graph& g, int k, size_t budget, const std::vector<uint8_t>& swap_of_tensor,
                const PlanOptions& opt, Plan* out, std::string* why);

// Three-stream discrete-event simulation of a plan (Algorithm 1 generalised: releases are
// modelled explicitly).  Fills t_ready / t_start / t_end / t_iter / t_stall.
void simulate(const Graph& g, const CostModel& cm, Plan* plan);

// Strategy search.  mode: ACC_PLAN_NONE / NAIVE_ALL / DYNAMIC.  Returns an acc_status.
int make_plan(const Graph& g, const CostModel& cm, int k, size_t budget, int mode, Plan* out,
              std::string* why);

// High-water mark of live dynamic bytes for a swap set with just-in-time allocation.
size_t live_peak(const Graph& g, int k, const std::vector<uint8_t>& swap_of_tensor);

}  // namespace acc
