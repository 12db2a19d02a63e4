#include "residency.h"

#include "gc3.h"
#include "program.h"

namespace gc3 {

int residency_waits(const std::vector<InFlightRun>& inflight, uint64_t stream, int32_t wgs, int32_t capacity,
                    std::vector<char>& wait_on) {
  wait_on.assign(inflight.size(), 0);
  auto share = [](int32_t w, int32_t cap) { return cap > 0 ? (double)w / (double)cap : 1.0; };
  double others = 0;
  for (const InFlightRun& r : inflight)
    if (r.stream != stream) others += share(r.wgs, r.capacity);
  const double mine = share(wgs, capacity);
  int marked = 0;
  for (size_t i = 0; i < inflight.size() && others + mine > 1.0 + 1e-9; ++i) {
    if (inflight[i].stream == stream) continue;
    wait_on[i] = 1;
    others -= share(inflight[i].wgs, inflight[i].capacity);
    ++marked;
  }
  return marked;
}

}  // namespace gc3

extern "C" int gc3_residency_plan(const gc3_inflight* inflight, int n, uint64_t stream, int32_t wgs, int32_t capacity,
                                  int32_t* wait_on) {
  if (n < 0 || (n > 0 && (!inflight || !wait_on)) || wgs < 0 || capacity < 1) {
    gc3::set_error("bad argument");
    return GC3_ERR_ARG;
  }
  std::vector<gc3::InFlightRun> runs;
  for (int i = 0; i < n; ++i) {
    if (inflight[i].wgs < 0 || inflight[i].capacity < 1) { gc3::set_error("bad ledger entry"); return GC3_ERR_ARG; }
    runs.push_back({inflight[i].stream, inflight[i].wgs, inflight[i].capacity});
  }
  std::vector<char> marks;
  const int marked = gc3::residency_waits(runs, stream, wgs, capacity, marks);
  for (int i = 0; i < n; ++i) wait_on[i] = marks[i];
  return marked;
}
