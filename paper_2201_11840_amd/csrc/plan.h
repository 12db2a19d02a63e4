// Execution plan of a program on a device of given size: flattened instruction tables, team
// width, which thread-block lanes share a workgroup, and workgroup placement.  Host only.
#pragma once
#include <string>
#include <vector>

#include "device_tables.h"
#include "program.h"

namespace gc3 {

struct Plan {
  gc3_comm_config cfg{};           // with defaults applied
  std::vector<DTb> tbs;
  std::vector<DInstr> instrs;
  std::vector<DDep> deps;
  std::vector<DWg> wgs;            // [grid], lane-major
  std::vector<DFiber> fibers;
  int nconn = 0, ntb = 0, max_count = 1;
  int max_pushes = 0;              // most send-type instructions in one thread block (messages per tile)
  uint64_t algorithmic_chunks = 0;
  gc3_comm_info info{};
};

// Apply defaults to `cfg_in` and check ranges.
int resolve_config(const gc3_comm_config* cfg_in, gc3_comm_config& cfg, std::string& msg);

// Validate `prog` and plan it for a device with `cus` compute units that can hold `resident`
// workgroups of cfg.wg_size threads at once.  `fifo_limit` = 0: the slot tile defaults to 64 KiB, halved (not
// below 16 KiB) while all FIFOs exceed 256 MiB.  `fifo_limit` > 0: a hard bound on the FIFO memory; the default
// tile is halved (not below 1 KiB) until the FIFOs fit, and a plan that still does not fit is GC3_ERR_SIZE.
int make_plan(const gc3_program& prog, const gc3_comm_config& cfg, int cus, long resident, Plan& plan, std::string& msg,
              uint64_t fifo_limit = 0);

}  // namespace gc3
