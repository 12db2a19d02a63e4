// Stand-alone use of the C ABI (no Python, no torch): load a GC3-IR program from a file, create a
// communicator, bind hipMalloc'ed buffers for every virtual rank, run, check.
//
//   python -m paper_2201_11840_amd.gc3c ring_allreduce --ranks 8 --instances 2 -o ring.gc3ir
//   hipcc --offload-arch=gfx950 -I include allreduce_c_abi.cpp -L paper_2201_11840_amd/lib -lgc3 -o allreduce_c_abi
//   ./allreduce_c_abi ring.gc3ir 1048576
//
// The program must be an in-place AllReduce; the buffers hold small integers (as floats), so every sum is
// exact and the result can be checked against the plain sum whatever the reduction order is.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "gc3.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define GC3_CHECK(x) do { int s_ = (x); if (s_ != GC3_OK) { std::fprintf(stderr, "%s: status %d: %s\n", #x, s_, gc3_last_error()); return 3; } } while (0)

int main(int argc, char** argv) {
  if (argc < 3) { std::fprintf(stderr, "usage: %s <program.gc3ir> <elements per rank>\n", argv[0]); return 1; }
  std::ifstream f(argv[1]);
  if (!f) { std::fprintf(stderr, "cannot read %s\n", argv[1]); return 1; }
  std::stringstream ss;
  ss << f.rdbuf();
  const std::string text = ss.str();
  const size_t elems = std::strtoull(argv[2], nullptr, 10);

  gc3_program* prog = nullptr;
  GC3_CHECK(gc3_program_load(text.data(), text.size(), &prog));
  gc3_program_info pi;
  GC3_CHECK(gc3_program_info_get(prog, &pi));
  if (!pi.inplace) { std::fprintf(stderr, "this example wants an in-place AllReduce program\n"); return 1; }

  gc3_comm_config cfg = {};                       // zero = defaults
  gc3_comm_config tuned = {};
  GC3_CHECK(gc3_comm_tune(prog, &cfg, elems, GC3_F32, nullptr, &tuned, nullptr));
  gc3_comm* comm = nullptr;
  GC3_CHECK(gc3_comm_create(prog, &tuned, &comm));
  gc3_comm_info ci;
  GC3_CHECK(gc3_comm_info_get(comm, &ci));

  const int R = pi.ranks;
  std::vector<float*> bufs(R, nullptr);
  std::vector<void*> scratch(R, nullptr);
  std::vector<float> host(elems), want(elems, 0.0f);
  for (int r = 0; r < R; ++r) {
    for (size_t i = 0; i < elems; ++i) {
      host[i] = (float)((long)((i * 2654435761u + 40503u * (unsigned)r) >> 7) % 17 - 8);   // integers in [-8, 8]
      want[i] += host[i];
    }
    HIP_OK(hipMalloc((void**)&bufs[r], elems * sizeof(float)));
    HIP_OK(hipMemcpy(bufs[r], host.data(), elems * sizeof(float), hipMemcpyHostToDevice));
    int sc = 0;
    GC3_CHECK(gc3_program_scratch_chunks(prog, r, &sc));
    const size_t sbytes = (size_t)sc * (elems / pi.in_chunks) * sizeof(float);
    if (sbytes) HIP_OK(hipMalloc(&scratch[r], sbytes));
    GC3_CHECK(gc3_comm_bind(comm, r, bufs[r], nullptr, scratch[r], sbytes));
  }
  gc3_program_free(prog);

  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  GC3_CHECK(gc3_comm_run(comm, elems, GC3_F32, GC3_SUM, stream));
  GC3_CHECK(gc3_comm_status(comm));

  size_t wrong = 0;
  for (int r = 0; r < R; ++r) {
    HIP_OK(hipMemcpy(host.data(), bufs[r], elems * sizeof(float), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < elems; ++i) wrong += host[i] != want[i];
  }
  uint64_t alg = 0;
  GC3_CHECK(gc3_comm_algorithmic_bytes(comm, elems, GC3_F32, &alg));
  std::printf("%s: %d ranks, %zu elements per rank, W=%d grid=%d: %s (%zu wrong), %llu algorithmic bytes\n", argv[1], R, elems,
              ci.team_width, ci.grid, wrong ? "MISMATCH" : "OK", wrong, (unsigned long long)alg);
  gc3_comm_destroy(comm);
  for (int r = 0; r < R; ++r) { (void)hipFree(bufs[r]); if (scratch[r]) (void)hipFree(scratch[r]); }
  (void)hipStreamDestroy(stream);
  return wrong ? 4 : 0;
}
