// Scratch memory of the entry point that allocates nothing (spd_decode_step_noalloc).
//
// Callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid it) get a decode step whose device-side working memory - the device twins of
// the step's metadata and the split-K partials - lies in one file-scope device array instead of
// buffers from hipMalloc.  Every GPU on which the library runs holds the array (SCRATCH_BYTES) from
// the moment the code object is loaded until the process ends.
//
// In host code the array's name is only a stand-in for the symbol: its device address is looked up
// once per device with hipGetSymbolAddress (here, called from spd_ctx_create with that device
// current) and only that address is handed to kernels and copies.
#include "internal.h"

namespace spd {

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

static std::mutex g_scratch_mu;
static std::map<int, char*> g_scratch_ptr;          // device ordinal -> address of that GPU's copy

int scratch_resolve(int device, char** out) {
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  auto it = g_scratch_ptr.find(device);
  if (it != g_scratch_ptr.end()) { *out = it->second; return SPD_OK; }
  int cur = -1;
  SPD_HIP(hipGetDevice(&cur));
  if (cur != device) SPD_HIP(hipSetDevice(device));
  void* ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (cur != device) (void)hipSetDevice(cur);
  if (e != hipSuccess) return hip_fail(e);
  if (!ptr || ((uintptr_t)ptr & 255) != 0) return SPD_ESTATE;
  g_scratch_ptr[device] = (char*)ptr;
  *out = (char*)ptr;
  return SPD_OK;
}

}  // namespace spd
