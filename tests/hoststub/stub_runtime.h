// Counters and controls of the host-only HIP stand-in (stub_runtime.cpp).  TEST INFRASTRUCTURE.
#pragma once
#include <hip/hip_runtime.h>

struct StubCounters {
  long events_created = 0, events_destroyed = 0, max_live_events = 0;
  long records = 0, stream_waits = 0, host_waits = 0, elapsed_reads = 0;
  long copies = 0, launches = 0, graph_launches = 0;
  unsigned long long copy_bytes = 0;
  // what must stay zero
  long dead_event_uses = 0, waits_on_unrecorded = 0, waits_on_stale = 0, elapsed_on_untimed = 0;
  long copies_out_of_range = 0, pointers_outside_pool = 0, null_streams = 0, sync_in_capture = 0;
  long waits_on_own_stream = 0;   // reported, not an error
  char first_complaint[160] = {0};
};
StubCounters& stub_counters();
void stub_set_regions(void* pool, size_t pool_bytes, void* arena, size_t arena_bytes);
void stub_new_epoch();            // call before every iteration: waits must find records of this epoch
hipStream_t stub_make_stream(int id);
void stub_free_stream(hipStream_t s);
long stub_live_events();
