// Which runs in flight a new run has to wait for so that every interpreter grid on the device stays resident.
//
// All workgroups of a run wait on each other (Section 6.2: the thread blocks of a program run concurrently),
// so a grid that is only partly resident never finishes.  One communicator checks its own grid against the
// device when it is created; two communicators launched on two streams could still be in flight together and
// exceed the device between them.  The library therefore keeps, per device, a ledger of the runs it has
// launched, and before launching another one makes its stream wait for earlier runs on OTHER streams until
// what may be in flight together fits.  This file holds the rule itself (host only, no device calls).
#pragma once
#include <cstdint>
#include <vector>

namespace gc3 {

struct InFlightRun {
  uint64_t stream;     // identity of the stream the run was launched on
  int32_t wgs;         // workgroups of the run
  int32_t capacity;    // workgroups of that size the device holds at once
};

// `inflight` in launch order (oldest first).  A run's share of the device is wgs / capacity.  Runs on `stream`
// itself are ordered before the new run by the stream and never overlap with it.  Marks in `wait_on` the
// runs the new one has to wait for: the oldest runs on other streams, as many as it takes for the shares of
// the rest plus the new run's to stay within the whole device.  Returns the number marked.
int residency_waits(const std::vector<InFlightRun>& inflight, uint64_t stream, int32_t wgs, int32_t capacity,
                    std::vector<char>& wait_on);

}  // namespace gc3
