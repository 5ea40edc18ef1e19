// fs_launch_static: fs_launch for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  A plan's scratch memory -- the
// partial rows of column reductions, the intermediates of a per-op plan -- comes from an array that is
// part of the library's device code instead of from a hipMalloc on the plan's first launch.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>
#include <string>

#include "../../include/fs.h"
#include "plan.h"

// One copy of this array exists on every GPU the library's code object is loaded on, from that moment
// until the process ends.  In host code its name is only a handle for hipGetSymbolAddress: the device
// address differs per GPU and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[FS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once asked for

// The array's address on the current device, asked once per device with that device current.
fs_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return fs::set_error(FS_ERR_HIP, "fs_launch_static: hipGetDevice failed");
  if (dev < 0 || dev >= kMaxDevices) return fs::set_error(FS_ERR_INVALID, "fs_launch_static: device ordinal out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fs::set_error(FS_ERR_HIP, std::string("fs_launch_static: hipGetSymbolAddress: ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FS_OK;
}

}  // namespace

extern "C" fs_status fs_launch_static(fs_plan* p, const void* const* inputs, int32_t n_in, void* const* outputs,
                                      int32_t n_out, void* hip_stream) {
  const fs_status st = fs::check_launch_args(p, inputs, n_in, outputs, n_out);
  if (st != FS_OK) return st;
  if (p->workspace_bytes > (int64_t)FS_STATIC_SCRATCH_BYTES) {
    char buf[160];
    snprintf(buf, sizeof buf, "fs_launch_static: the plan needs %lld bytes of scratch memory, the static array holds %lld",
             (long long)p->workspace_bytes, (long long)FS_STATIC_SCRATCH_BYTES);
    return fs::set_error(FS_ERR_UNSUPPORTED, buf);
  }
  // a generated kernel is put on the device by the plan's first fs_launch; loading a code object allocates
  const bool elementwise = p->schedule == FS_SCHED_ELEMENTWISE;
  const bool generated = elementwise ? p->ew.generated : (p->schedule != FS_SCHED_PER_OP && p->row_form == 3);
  const fs::EwModule& mod = elementwise ? p->ew.loaded : p->row_gen.loaded;
  int dev = -1;
  if (generated && (hipGetDevice(&dev) != hipSuccess || !mod.function || mod.device != dev))
    return fs::set_error(FS_ERR_INVALID, "fs_launch_static: this plan runs a generated kernel that is not on this device yet; "
                                         "launch it once with fs_launch (or build the plan with FS_MODE_STITCHED_PREBUILT)");
  void* ws = nullptr;
  if (p->workspace_bytes > 0) {
    // Nothing in the array has to start at zero: every kernel that reads scratch memory reads only what
    // an earlier kernel of the same call wrote there.
    const fs_status s2 = static_scratch(&ws);
    if (s2 != FS_OK) return s2;
  }
  return fs::enqueue_plan(p, inputs, outputs, n_out, ws, hip_stream);
}
