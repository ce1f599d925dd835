// Optional per-kernel timing with HIP events on the launch stream, for benchmarks.
// Off by default; when off a launch costs one predictable branch.  Not thread-safe:
// enable, run and read from one host thread.
#include <vector>

#include "../../include/vector.h"
#include "launch.hpp"

namespace vec {

namespace {
struct Span { hipEvent_t start, stop; };
struct Slot {
  std::vector<Span> spans;     // recorded since the last read
  std::vector<Span> free_list; // events ready for reuse
};
bool g_enabled = false;
Slot g_slots[K_COUNT];
const char* const kNames[K_COUNT] = {"score_stats", "stats_combine", "mass_residual", "pool_scores",
                                     "route", "gather_rows", "decode_split", "decode_combine"};
}  // namespace

bool timing_enabled() { return g_enabled; }

void timing_begin(int id, hipStream_t stream) {
  Slot& s = g_slots[id];
  Span sp;
  if (!s.free_list.empty()) {
    sp = s.free_list.back();
    s.free_list.pop_back();
  } else {
    if (hipEventCreate(&sp.start) != hipSuccess || hipEventCreate(&sp.stop) != hipSuccess) return;
  }
  hipEventRecord(sp.start, stream);
  s.spans.push_back(sp);
}

void timing_end(int id, hipStream_t stream) {
  Slot& s = g_slots[id];
  if (!s.spans.empty()) hipEventRecord(s.spans.back().stop, stream);
}

}  // namespace vec

extern "C" {

int vector_timing_enable(int on) {
  vec::g_enabled = on != 0;
  return VECTOR_OK;
}

int vector_timing_kernels(void) { return vec::K_COUNT; }

const char* vector_timing_name(int kernel_id) {
  return (kernel_id >= 0 && kernel_id < vec::K_COUNT) ? vec::kNames[kernel_id] : "";
}

int vector_timing_read(int kernel_id, double* total_ms, int64_t* launches) {
  if (kernel_id < 0 || kernel_id >= vec::K_COUNT || !total_ms || !launches) return VECTOR_ERR_ARG;
  vec::Slot& s = vec::g_slots[kernel_id];
  double sum = 0.0;
  int64_t count = 0;
  for (vec::Span& sp : s.spans) {
    if (hipEventSynchronize(sp.stop) != hipSuccess) return VECTOR_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, sp.start, sp.stop) != hipSuccess) return VECTOR_ERR_HIP;
    sum += ms;
    ++count;
    s.free_list.push_back(sp);
  }
  s.spans.clear();
  *total_ms = sum;
  *launches = count;
  return VECTOR_OK;
}

}  // extern "C"
