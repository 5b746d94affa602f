// Runs the library's host-side spec parser and planner (fbx_plan.cpp, no HIP involved) on the spec
// files given on the command line, for a build with -fsanitize=address,undefined
// (test infrastructure: see tests/test_host_sanitizers.py).
#include <cstdio>
#include <fstream>
#include <sstream>
#include <string>

#include "fbx_internal.h"

int main(int argc, char** argv) {
  for (int i = 1; i < argc; ++i) {
    std::ifstream f(argv[i], std::ios::binary);
    std::stringstream ss;
    ss << f.rdbuf();
    const std::string spec = ss.str();
    fbx::PlanHost plan;
    std::string err;
    const fbx_status st = fbx::parse_plan(spec.data(), spec.size(), plan, err);
    std::printf("%s: status %d, %zu operators, %u layers, %u ragged%s%s\n", argv[i], (int)st, plan.ops.size(), plan.n_layers,
                plan.n_ragged, err.empty() ? "" : " -- ", err.c_str());
  }
  return 0;
}
