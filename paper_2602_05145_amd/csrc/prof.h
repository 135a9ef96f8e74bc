// Optional per-launch timing of the library's kernels with HIP events recorded on the caller's stream
// (switched on by tide_profile_start; costs one branch per launch when off).
#pragma once
#include <hip/hip_runtime.h>

namespace tide {

bool prof_enabled();
void prof_begin(const char* kernel, double flops, double bytes, hipStream_t s);
// the launch just begun works on clamp(*dev - off, 0, maxv) of the maxv units its flops/bytes were computed for
void prof_dynamic(const int* dev, long long off, long long maxv);
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
