// Event-based per-kernel timing (benchmark aid).
#include <hip/hip_runtime.h>

#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "mux_internal.h"

namespace mux {
namespace {
struct Rec { const char* name; hipEvent_t a, b; double bytes; };
int g_on = 0;            // 0 off, 1 every kernel, 2 backbone GEMM kernels only
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
hipEvent_t g_open = nullptr;
const char* g_open_name = nullptr;
unsigned long long* g_clock = nullptr;
double g_next_bytes = 0.0;

hipEvent_t get_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

unsigned long long* diag_clock_buffer() { return g_clock; }

void prof_note_bytes(double bytes) { g_next_bytes = bytes; }

void prof_begin(const char* name, hipStream_t stream) {
  if (!g_on) return;
  if (g_on == 2 && std::strncmp(name, "gemm", 4) != 0) return;
  g_open = get_event();
  g_open_name = name;
  if (g_open) (void)hipEventRecord(g_open, stream);
}

void prof_end(hipStream_t stream) {
  const double bytes = g_next_bytes;
  g_next_bytes = 0.0;                    // a note covers one launch, bracketed or not
  if (!g_on || !g_open) return;
  hipEvent_t b = get_event();
  if (b) {
    (void)hipEventRecord(b, stream);
    g_recs.push_back({g_open_name, g_open, b, bytes});
  } else {
    g_pool.push_back(g_open);
  }
  g_open = nullptr;
}
}  // namespace mux

using namespace mux;

extern "C" mux_status mux_diag_set_clock_buffer(void* dev_four_u64) {
  if (((uintptr_t)dev_four_u64 & 7) != 0) return fail(MUX_ERR_INVALID_ARG, "mux_diag_set_clock_buffer: the buffer must be 8-byte aligned");
  g_clock = (unsigned long long*)dev_four_u64;
  return MUX_OK;
}

extern "C" mux_status mux_profile_enable(int on) {
  if (on < 0 || on > 2) return fail(MUX_ERR_INVALID_ARG, "mux_profile_enable: mode must be 0, 1 or 2");
  g_on = on;
  return MUX_OK;
}

extern "C" mux_status mux_profile_collect(mux_profile_entry* out, int32_t cap, int32_t* n) {
  if (!n || cap < 0 || (cap > 0 && !out)) return fail(MUX_ERR_INVALID_ARG, "mux_profile_collect: bad argument");
  std::vector<const char*> order;
  std::map<const char*, std::pair<int, double>> sum;
  std::map<const char*, double> bytes;
  mux_status st = MUX_OK;
  for (const Rec& r : g_recs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) st = fail(MUX_ERR_DEVICE, std::string("mux_profile_collect: ") + hipGetErrorString(e));
    if (!sum.count(r.name)) order.push_back(r.name);
    sum[r.name].first += 1;
    sum[r.name].second += ms;
    bytes[r.name] += r.bytes;
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_recs.clear();
  *n = (int32_t)order.size();
  for (int32_t i = 0; i < (int32_t)order.size() && i < cap; ++i) {
    out[i].name = order[i];
    out[i].launches = sum[order[i]].first;
    out[i].total_ms = sum[order[i]].second;
    out[i].bytes = bytes[order[i]];
  }
  return st;
}
