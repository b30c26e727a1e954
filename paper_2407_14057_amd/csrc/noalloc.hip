// Eq. 1 scoring for callers that cannot allocate: the same three kernels as lazyllm_op_score,
// with their scratch (logits, per-workgroup partial statistics, per-head statistics) in a
// file-scope device array instead of a caller-provided buffer.  No hipMalloc / hipFree, no
// allocating library routine, no host synchronisation.
#include <mutex>

#include "../../include/lazyllm.h"
#include "common.h"

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress: the address a
// kernel may use is the one that call returns on the device in question.
constexpr size_t kScratchBytes = LAZYLLM_SCORE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch`, per device ordinal
bool g_scratch_known[kMaxDevices];

// The device address of this device's copy of `scratch`; looked up once per device, with that
// device current (it is: the ordinal comes from hipGetDevice).
hipError_t scratch_for_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_known[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
    g_scratch_known[dev] = true;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" {

int lazyllm_op_score_static(const void* q_last, const void* k, float* s, int32_t rows,
                            int32_t n_heads, int32_t head_dim, void* hip_stream) {
  // the same argument rules as lazyllm_op_score, checked before any HIP call
  if (!q_last || !k || !s || rows <= 0 || n_heads <= 0 || n_heads > 256 ||
      (head_dim != 64 && head_dim != 128) || (n_heads * head_dim) % 8 != 0 ||
      n_heads * head_dim > 8192)
    return LAZYLLM_EINVAL;
  // sizes beyond the static array are refused, never truncated
  if (lz::score_scratch_bytes(rows, 1, n_heads) > kScratchBytes) return LAZYLLM_ENOSPC;
  void* ptr = nullptr;
  hipError_t e = scratch_for_current_device(&ptr);
  if (e != hipSuccess) {
    lz::set_last_hip_error((int)e);
    return LAZYLLM_EHIP;
  }
  // Nothing in the scratch has to start at zero: every logit, partial and statistic that a launch
  // reads was written by an earlier kernel of the same call (rows and partials beyond this call's
  // sizes are never read), so the contents a previous, larger call left behind are harmless.
  const char* qbase = (const char*)q_last - (size_t)(rows - 1) * n_heads * head_dim * 2;
  e = lz::launch_score(qbase, k, s, ptr, nullptr, rows, 1, rows, rows, n_heads, head_dim,
                       (hipStream_t)hip_stream);
  if (e != hipSuccess) {
    lz::set_last_hip_error((int)e);
    return LAZYLLM_EHIP;
  }
  return LAZYLLM_OK;
}

}  // extern "C"
