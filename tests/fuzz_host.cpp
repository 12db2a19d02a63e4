// Host-only robustness driver for the IR loader, validator and planner (no device code): reads seed programs
// from the files named on the command line, mutates them at random (bytes, tokens, numbers, lines) and feeds
// every mutant to gc3_program_load / gc3_program_validate / gc3_program_plan.  Built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_library.py; any status is fine, a crash or a sanitizer report is not.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "gc3.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {                       // xorshift64*
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return rng_state * 0x2545F4914F6CDD1Dull;
}

static std::string mutate(const std::string& src) {
  std::string s = src;
  const int n = 1 + (int)(rnd() % 4);
  const bool gentle = rnd() & 1;   // half of the mutants only change digits: the text still parses and the
                                   // validator and planner see wrong indices, peers, counts and dependencies
  for (int k = 0; k < n && !s.empty(); ++k) {
    size_t pos = rnd() % s.size();
    if (gentle) {
      for (size_t tries = 0; tries < s.size() && !(s[pos] >= '0' && s[pos] <= '9'); ++tries) pos = (pos + 1) % s.size();
    }
    switch (gentle ? 6 : rnd() % 7) {
      case 0: s[pos] = (char)(rnd() & 0xff); break;                                     // random byte
      case 1: s.erase(pos, 1 + rnd() % 8); break;                                       // drop a few bytes
      case 2: s.insert(pos, std::to_string((long long)(rnd() % 7) - 3)); break;         // stray small number
      case 3: s.insert(pos, std::to_string(rnd())); break;                              // huge number
      case 4: { size_t e = s.find('\n', pos); if (e != std::string::npos) s.erase(pos, e - pos); break; }   // cut a line short
      case 5: { size_t b = s.rfind('\n', pos), e = s.find('\n', pos);                   // duplicate a line
                if (b != std::string::npos && e != std::string::npos) s.insert(e, s.substr(b, e - b)); break; }
      default: if (s[pos] >= '0' && s[pos] <= '9') s[pos] = (char)('0' + rnd() % 10); break;   // change a digit
    }
  }
  return s;
}

int main(int argc, char** argv) {
  if (argc < 3) { std::fprintf(stderr, "usage: %s <iterations> <program files...>\n", argv[0]); return 2; }
  const long iters = std::strtol(argv[1], nullptr, 10);
  std::vector<std::string> seeds;
  for (int i = 2; i < argc; ++i) {
    std::ifstream f(argv[i]);
    std::stringstream ss;
    ss << f.rdbuf();
    seeds.push_back(ss.str());
  }
  long loaded = 0, valid = 0, planned = 0;
  for (long it = 0; it < iters; ++it) {
    const std::string text = it < (long)seeds.size() ? seeds[it] : mutate(seeds[rnd() % seeds.size()]);
    gc3_program* p = nullptr;
    if (gc3_program_load(text.data(), text.size(), &p) != GC3_OK) continue;
    ++loaded;
    char err[128];
    const int slots = 1 + (int)(rnd() % 8);
    if (gc3_program_validate(p, slots, err, sizeof err) == GC3_OK) {
      ++valid;
      gc3_comm_config cfg = {};
      cfg.fifo_slots = slots;
      cfg.team_width = (int)(rnd() % 5) * (int)(rnd() % 9);
      cfg.target_wgs = (int)(rnd() % 3) * 300;
      gc3_comm_info info;
      if (gc3_program_plan(p, &cfg, 256, 1792, &info) == GC3_OK) ++planned;
    }
    gc3_program_info pi;
    (void)gc3_program_info_get(p, &pi);
    for (int r = -1; r <= pi.ranks; ++r) { int sc; (void)gc3_program_scratch_chunks(p, r, &sc); }
    gc3_program_free(p);
  }
  std::printf("%ld inputs: %ld parsed, %ld valid, %ld planned\n", iters, loaded, valid, planned);
  return (loaded >= (long)seeds.size() && planned >= (long)seeds.size()) ? 0 : 1;
}
