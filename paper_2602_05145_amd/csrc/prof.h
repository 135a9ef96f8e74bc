// Optional per-launch timing of the library's kernels with HIP events recorded on the caller's stream
// (switched on by tide_profile_start; costs one branch per launch when off).
#pragma once
#include <hip/hip_runtime.h>

namespace tide {

bool prof_enabled();
void prof_begin(const char* kernel, double flops, double bytes, hipStream_t s);
void prof_end(hipStream_t s);

struct ProfScope {
  hipStream_t s;
  bool on;
  ProfScope(const char* kernel, double flops, double bytes, hipStream_t stream) : s(stream), on(prof_enabled()) {
    if (on) prof_begin(kernel, flops, bytes, s);
  }
  ~ProfScope() {
    if (on) prof_end(s);
  }
};

}  // namespace tide
