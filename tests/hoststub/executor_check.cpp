// Drives the real planner and executor (graph.cpp, plan.cpp, engine.hip built for the host
// against the stand-in runtime beside this file) through whole iterations and prints what the
// stand-in counted.  usage: executor_check <spec.bin> <scenario>
//   spec.bin: int32 n_layers, in_c, in_h, in_w, then n_layers records of 9 int32
//   scenario "timed_swap_all": ResNet-sized plans that swap every map at minibatch 224 and 256
//            under 8 GiB, event timing of every step, copy and kernel on (level 3), re-planned
//            between iterations - the combination that is refused on the GPU; here the limit
//            is lifted at compile time
//   scenario "guard": the same plan with the limit in place must be refused before anything
//            is issued
//   scenario "dynamic": planner-chosen swaps at minibatch 64, untimed and timed, weight
//            gradients on their own stream
// TEST INFRASTRUCTURE.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/accudnn.h"
#include "stub_runtime.h"

static int fail(const char* what, acc_ctx* c) {
  printf("FAILED %s: %s\n", what, c ? acc_last_error(c) : acc_last_error(nullptr));
  return 1;
}

int main(int argc, char** argv) {
  if (argc < 3) return 2;
  FILE* f = fopen(argv[1], "rb");
  if (!f) return 2;
  int32_t hdr[4];
  if (fread(hdr, 4, 4, f) != 4) return 2;
  std::vector<acc_layer> layers(hdr[0]);
  if (fread(layers.data(), sizeof(acc_layer), layers.size(), f) != layers.size()) return 2;
  fclose(f);
  const std::string scenario = argv[2];

  const size_t GiB = (size_t)1 << 30;
  const size_t budget = 8 * GiB, arena = 64 * GiB;
  // address ranges nobody dereferences: the stand-in only checks that copies and kernel
  // operands stay inside them
  void* pool = (void*)(uintptr_t)0x500000000000ull;
  void* host = (void*)(uintptr_t)0x600000000000ull;
  stub_set_regions(pool, budget, host, arena);
  hipStream_t st[4];
  for (int i = 0; i < 4; ++i) st[i] = stub_make_stream(i);
  acc_resources res{pool, budget, host, arena, st[0], st[1], st[2], st[3]};
  acc_ctx* c = nullptr;
  if (acc_create(layers.data(), (int)layers.size(), hdr[1], hdr[2], hdr[3], ACC_F32, &res, &c) != ACC_OK) return fail("create", nullptr);
  std::vector<int32_t> labels(512, 1);
  const float* images = (const float*)(uintptr_t)0x700000000000ull;   // never read by the stand-in
  float loss = 0.f;
  int rc = 0;
  auto steps = [&](int n, const char* what) {
    for (int i = 0; i < n && !rc; ++i) {
      stub_new_epoch();
      if (acc_train_step(c, images, ACC_LOC_HOST, labels.data(), 0.1f, &loss) != ACC_OK) rc = fail(what, c);
    }
  };
  acc_plan_summary s;
  if (scenario == "timed_swap_all") {
    for (int round = 0; round < 2 && !rc; ++round)
      for (int k : {224, 256, 64}) {
        if (acc_plan_swaps(c, k, budget, ACC_PLAN_NAIVE_ALL, &s) != ACC_OK) { rc = fail("plan", c); break; }
        acc_set_profiling(c, 3);
        steps(2, "timed step");
        acc_set_profiling(c, 1);
        steps(1, "timed step, level 1");
        acc_set_profiling(c, 0);
        steps(1, "untimed step");
        acc_timeline_entry* tl = new acc_timeline_entry[s.n_instr];
        acc_set_profiling(c, 1);
        steps(1, "timed step before the timeline");
        if (!rc && acc_get_timeline(c, 1, tl, s.n_instr) != s.n_instr) rc = fail("timeline", c);
        delete[] tl;
        printf("k=%d swapped %d maps, %.2f GiB each way, %d instructions\n", k, s.n_swapped, s.bytes_swapped / (double)GiB, s.n_instr);
        if (rc) break;
      }
  } else if (scenario == "guard") {
    if (acc_plan_swaps(c, 256, budget, ACC_PLAN_NAIVE_ALL, &s) != ACC_OK) rc = fail("plan", c);
    const StubCounters before = stub_counters();
    acc_set_profiling(c, 1);
    stub_new_epoch();
    const int r = acc_train_step(c, images, ACC_LOC_HOST, labels.data(), 0.1f, &loss);
    const StubCounters& after = stub_counters();
    printf("guard: status %d (ACC_ESTATE is %d), text: %s\n", r, ACC_ESTATE, acc_last_error(c));
    printf("guard: issued records %ld copies %ld launches %ld events %ld\n", after.records - before.records,
           after.copies - before.copies, after.launches - before.launches, after.events_created - before.events_created);
    if (r != ACC_ESTATE || after.records != before.records || after.copies != before.copies ||
        after.launches != before.launches || after.events_created != before.events_created) rc = 1;
    acc_set_profiling(c, 0);
    steps(1, "untimed step of the same plan");      // ... and runs untimed
  } else if (scenario == "dynamic") {
    if (acc_plan_swaps(c, 64, budget, ACC_PLAN_DYNAMIC, &s) != ACC_OK) rc = fail("plan", c);
    steps(2, "untimed step");
    acc_set_profiling(c, 3);
    steps(2, "timed step");
    acc_set_wgrad_overlap(c, 0);
    acc_set_profiling(c, 0);
    steps(1, "serial step");
    printf("k=64 swapped %d of %d maps\n", s.n_swapped, s.n_maps);
  } else if (scenario == "graph") {
    // an iteration that swaps nothing, recorded into a graph on its first run and replayed afterwards;
    // a new plan discards the recording; profiling runs the ordinary way in between
    acc_set_graph(c, 1);
    for (int k : {32, 41}) {
      if (acc_plan_swaps(c, k, budget, ACC_PLAN_DYNAMIC, &s) != ACC_OK) { rc = fail("plan", c); break; }
      if (s.n_swapped != 0) { rc = fail("expected a plan without swaps", c); break; }
      const long l0 = stub_counters().launches, g0 = stub_counters().graph_launches;
      steps(1, "capturing step");
      const long l1 = stub_counters().launches;
      steps(3, "replayed step");
      const long l2 = stub_counters().launches, g2 = stub_counters().graph_launches;
      printf("k=%d: capture issued %ld launches, three replays %ld launches and %ld graph launches in all\n", k, l1 - l0, l2 - l1, g2 - g0);
      if (g2 - g0 != 4 || l2 - l1 != 3) rc = 1;          // per replay: the graph and the update kernel
      acc_set_profiling(c, 1);
      steps(1, "timed step beside the recording");
      acc_set_profiling(c, 0);
      steps(1, "replayed step after a timed one");
      if (stub_counters().graph_launches - g2 != 1) rc = 1;
    }
    if (!rc && acc_plan_swaps(c, 64, budget, ACC_PLAN_DYNAMIC, &s) == ACC_OK) {
      const long g0 = stub_counters().graph_launches;
      steps(2, "swapping step with graph mode on");
      if (stub_counters().graph_launches != g0) rc = 1;  // plans that swap never use the graph
    }
  } else if (scenario == "selftest") {
    // the stand-in must see planted mistakes: a wait on an event nobody recorded, a wait on last
    // iteration's record, a timing read on an untimed event, a copy that leaves the pool
    hipEvent_t never, old, untimed;
    hipEventCreate(&never); hipEventCreate(&old); hipEventCreateWithFlags(&untimed, hipEventDisableTiming);
    hipEventRecord(old, st[0]);
    stub_new_epoch();
    hipEventRecord(untimed, st[0]);
    hipStreamWaitEvent(st[1], never, 0);
    hipStreamWaitEvent(st[1], old, 0);
    float ms;
    hipEventElapsedTime(&ms, untimed, untimed);
    hipMemcpyAsync((char*)pool + budget - 16, host, 64, hipMemcpyHostToDevice, st[2]);
    hipEventDestroy(never); hipEventDestroy(old); hipEventDestroy(untimed);
    const StubCounters& g = stub_counters();
    const bool seen = g.waits_on_unrecorded == 1 && g.waits_on_stale == 1 && g.elapsed_on_untimed == 1 && g.copies_out_of_range == 1;
    printf("selftest: unrecorded %ld stale %ld untimed %ld out of range %ld\n", g.waits_on_unrecorded, g.waits_on_stale,
           g.elapsed_on_untimed, g.copies_out_of_range);
    acc_destroy(c);
    for (int i = 0; i < 4; ++i) stub_free_stream(st[i]);
    printf(seen ? "RESULT: planted mistakes seen\n" : "RESULT: planted mistakes missed\n");
    return seen ? 0 : 1;
  } else {
    rc = 2;
  }
  acc_destroy(c);
  const StubCounters& g = stub_counters();
  printf("events created %ld destroyed %ld live now %ld max live %ld | records %ld stream waits %ld host waits %ld elapsed %ld | "
         "copies %ld (%.1f GiB) launches %ld\n",
         g.events_created, g.events_destroyed, stub_live_events(), g.max_live_events, g.records, g.stream_waits, g.host_waits,
         g.elapsed_reads, g.copies, g.copy_bytes / (double)GiB, g.launches);
  printf("violations: dead_event_uses %ld waits_on_unrecorded %ld waits_on_stale %ld elapsed_on_untimed %ld copies_out_of_range %ld "
         "pointers_outside_pool %ld null_streams %ld sync_in_capture %ld leaked_events %ld (waits on own stream: %ld)\n",
         g.dead_event_uses, g.waits_on_unrecorded, g.waits_on_stale, g.elapsed_on_untimed, g.copies_out_of_range,
         g.pointers_outside_pool, g.null_streams, g.sync_in_capture, stub_live_events(), g.waits_on_own_stream);
  if (g.first_complaint[0]) printf("first complaint: %s\n", g.first_complaint);
  const long bad = g.dead_event_uses + g.waits_on_unrecorded + g.waits_on_stale + g.elapsed_on_untimed + g.copies_out_of_range +
                   g.pointers_outside_pool + g.null_streams + g.sync_in_capture + stub_live_events();
  for (int i = 0; i < 4; ++i) stub_free_stream(st[i]);
  if (rc) return rc;
  printf(bad ? "RESULT: violations\n" : "RESULT: clean\n");
  return bad ? 1 : 0;
}
