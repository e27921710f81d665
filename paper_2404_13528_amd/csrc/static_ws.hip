// sm_swin_block_static: sm_swin_block for callers that cannot hand over a workspace they allocated (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The block's workspace (activation
// buffers and the per-row offset tables of its index maps) is a static device array of the library instead.
#include <hip/hip_runtime.h>
#include <mutex>
#include "common.h"

// One copy per GPU the library runs on, held until the process ends.
static __device__ __align__(256) unsigned char scratch[SM_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, asked for once per device
}

extern "C" size_t sm_swin_block_static_max_bytes(void) { return (size_t)SM_STATIC_WS_BYTES; }

extern "C" int sm_swin_block_static(const sm_swin_cfg* c, const sm_swin_weights* wt, const void* x, void* y, int mode, void* stream) {
  const size_t need = sm_swin_block_workspace_bytes(c, mode);        // validates c and mode; host work only
  if (need == 0) return SM_ERR_INVALID_ARG;                          // (message left by the query)
  if (need > (size_t)SM_STATIC_WS_BYTES)
    return sm::fail(SM_ERR_WORKSPACE, "sm_swin_block_static: this block needs %zu bytes of workspace, the static buffer holds %zu; "
                    "use sm_swin_block with a workspace of your own", need, (size_t)SM_STATIC_WS_BYTES);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return sm::fail(SM_ERR_DEVICE, "sm_swin_block_static: no current device");
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));       // this device's copy of the array
      if (e != hipSuccess || !p) return sm::fail(SM_ERR_DEVICE, "sm_swin_block_static: hipGetSymbolAddress failed (hip error %d)", (int)e);
      g_scratch_ptr[dev] = p;
    }
    ws = g_scratch_ptr[dev];
  }
  // nothing in the workspace has to start at zero: every call rewrites the tables and buffers it reads
  return sm_swin_block(c, wt, x, y, ws, (size_t)SM_STATIC_WS_BYTES, mode, stream);
}
