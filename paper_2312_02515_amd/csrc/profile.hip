// Optional per-launch timing of the MFMA kernels with HIP events recorded on the launch stream.
// A measurement aid (the benchmark's roofline figures come from here); off by default.
#include <mutex>
#include <vector>

#include "mlora_common.h"

namespace mlora {
namespace {

struct Record {
  hipEvent_t start, stop;
  int kind;
  double units;
};
struct Profile {
  bool on = false;
  std::vector<Record> rec;   // the first `used` entries hold launches not read yet
  size_t used = 0;
};
Profile g_prof;
std::mutex g_mu;
constexpr size_t kMaxProfiled = 16384;

}  // namespace

int profile_enable(int enable) {
  std::lock_guard<std::mutex> lk(g_mu);
  const int old = g_prof.on ? 1 : 0;
  g_prof.on = enable != 0;
  return old;
}

// Records the start event of a launch of kind `kind` doing `units` algorithmic units (flops for
// the base product, bytes for the low-rank kernels); returns its slot, or -1 when profiling is off.
int profile_begin(int kind, double units, hipStream_t stream) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_prof.on || g_prof.used >= kMaxProfiled) return -1;
  if (g_prof.used == g_prof.rec.size()) {
    Record r;
    if (hipEventCreate(&r.start) != hipSuccess) return -1;
    if (hipEventCreate(&r.stop) != hipSuccess) {
      (void)hipEventDestroy(r.start);
      return -1;
    }
    g_prof.rec.push_back(r);
  }
  const int slot = (int)g_prof.used++;
  g_prof.rec[slot].kind = kind;
  g_prof.rec[slot].units = units;
  (void)hipEventRecord(g_prof.rec[slot].start, stream);
  return slot;
}

void profile_end(int slot, hipStream_t stream) {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  (void)hipEventRecord(g_prof.rec[slot].stop, stream);
}

// Waits for every recorded launch, sums durations and units of the launches of each kind
// (arrays of kProfileKinds entries), then forgets all of them.
hipError_t profile_read(double* ms, double* units, int* launches) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (int k = 0; k < kProfileKinds; ++k) {
    ms[k] = 0;
    units[k] = 0;
    launches[k] = 0;
  }
  for (size_t i = 0; i < g_prof.used; ++i) {
    const Record& r = g_prof.rec[i];
    hipError_t e = hipEventSynchronize(r.stop);
    if (e != hipSuccess) return e;
    float t = 0.f;
    e = hipEventElapsedTime(&t, r.start, r.stop);
    if (e != hipSuccess) return e;
    ms[r.kind] += t;
    units[r.kind] += r.units;
    launches[r.kind] += 1;
  }
  g_prof.used = 0;
  return hipSuccess;
}

}  // namespace mlora
