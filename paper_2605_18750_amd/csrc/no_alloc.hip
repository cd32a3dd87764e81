// RMSNorm backward for callers that cannot allocate or pass a workspace: the partial gain-gradient rows
// live in a file-scope device array instead of caller memory.  Same kernels as rrfp_rmsnorm_bwd; the
// array is handed to them as an ordinary pointer argument.
#include <mutex>

#include "../../include/rrfp_kernels.h"
#include "../../include/rrfp_stage.h"
#include "kernels.h"

using namespace rrfp;

namespace {

constexpr size_t SCRATCH_BYTES = (size_t)16 << 20;   // 16 MiB per device, held until the process ends
constexpr int MAX_DEVICES = 64;

// Every device the library runs on holds its own copy of this array at its own address.  In host code the
// name is only a handle for hipGetSymbolAddress: it is never passed to a kernel or a memory call.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

std::mutex g_lock;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device; looked up once per device.
hipError_t scratch_ptr(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" size_t rrfp_rmsnorm_bwd_static_limit(void) { return SCRATCH_BYTES; }

extern "C" int rrfp_rmsnorm_bwd_static(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                                       float* out32, void* out_t, float* dg, int T, int H, int dtype, void* stream) {
  if (!dh || !x || !r || !g || !add_in || !dg || T < 1 || H < 1) return STAGE_EINVAL;
  if (dtype != F32 && dtype != BF16) return STAGE_EINVAL;
  const size_t need = rrfp_rmsnorm_bwd_workspace(T, H, dtype);
  if (need == 0 || need > SCRATCH_BYTES) return STAGE_ENOMEM;
  void* ws = nullptr;
  if (scratch_ptr(&ws) != hipSuccess) return STAGE_EHIP;
  hipStream_t s = (hipStream_t)stream;
  // every partial row the column sum reads is written by the first kernel of this call: nothing to clear
  if (launch_rmsnorm_bwd(dh, x, r, g, add_in, out32, out_t, (float*)ws, T, H, dtype, s) != hipSuccess) return STAGE_EHIP;
  if (launch_colsum((const float*)ws, norm_bwd_partials(T, H, dtype), H, dg, s) != hipSuccess) return STAGE_EHIP;
  return STAGE_OK;
}
