// Device-side sleep on a stream: the compute-path delay of the jitter protocol (Sec. 7.6), as a
// one-wavefront kernel that polls the constant-rate wall clock.  The poll count is bounded, so every
// wavefront reaches its exit whatever the clock does.
#include <hip/hip_runtime.h>

#include <string>

#include "../../include/rrfp_arbiter.h"

namespace {

__global__ __launch_bounds__(64) void delay_kernel(unsigned long long ticks, unsigned long long max_polls) {
  const unsigned long long t0 = wall_clock64();
  for (unsigned long long i = 0; i < max_polls; ++i) {
    if (wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(16);
  }
}

thread_local std::string g_delay_error;

}  // namespace

extern "C" const char* rrfp_delay_last_error() { return g_delay_error.c_str(); }

extern "C" int rrfp_delay(double seconds, void* stream) {
  if (!(seconds >= 0.0) || seconds > 1.0) { g_delay_error = "rrfp_delay: seconds must be in [0, 1]"; return ARB_EINVAL; }
  int dev = 0, khz = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
  if (e != hipSuccess || khz <= 0) {
    g_delay_error = std::string("rrfp_delay: ") + (e != hipSuccess ? hipGetErrorString(e) : "wall clock rate unknown");
    return ARB_ESTATE;
  }
  const unsigned long long ticks = (unsigned long long)(seconds * 1e3 * (double)khz);
  // a poll takes at least the s_sleep (16 x 64 clocks, > 0.25 us at any clock the part runs at): 8 polls
  // per requested microsecond plus slack bound the kernel to a small multiple of the request
  const unsigned long long max_polls = (unsigned long long)(seconds * 8e6) + 4096;
  hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, ticks, max_polls);
  e = hipGetLastError();
  if (e != hipSuccess) { g_delay_error = std::string("rrfp_delay: ") + hipGetErrorString(e); return ARB_ESTATE; }
  return ARB_OK;
}
