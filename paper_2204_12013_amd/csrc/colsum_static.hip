// bk_colsum_acc_static: the column-sum entry point for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// bk_colsum_acc takes its partial-row buffer from the caller; here the partial rows live in a
// file-scope device array instead, so the call needs nothing beyond its input and its output.  Each
// GPU the library runs on holds its own copy of the array (kStaticFloats * 4 bytes = 2 MiB) until the
// process ends.  The array's name is a host-side stand-in, not a device address: the device address is
// looked up once per device with hipGetSymbolAddress and only that pointer is handed to the kernels.
#include <mutex>

#include "../../include/bamboo_kernels.h"
#include "../../include/bamboo_stage.h"
#include "common.h"

using namespace bamboo;

namespace {

constexpr size_t kStaticFloats = 512 * 1024;    // partial rows x columns that one call may need
constexpr int kMaxDevices = 64;

static __device__ __align__(256) float scratch[kStaticFloats];

std::mutex g_lock;
float* g_scratch_ptr[kMaxDevices];              // per device: address of that GPU's copy of `scratch`

// Address of the current device's copy of the array; looked up on the first call on that device.
int scratch_for_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return BAMBOO_E_HIP;
  }
  std::lock_guard<std::mutex> hold(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return BAMBOO_E_HIP;
    }
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return BAMBOO_OK;
}

}  // namespace

extern "C" {

uint64_t bk_colsum_static_max_floats(void) { return kStaticFloats; }

int bk_colsum_acc_static(int dtype, int T, int N, const void* A, float* out, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || N <= 0 || N % 2 || !A || !out) return BAMBOO_E_ARG;
  // the partial rows this shape produces must fit the array: rejected here, before anything is launched
  const int rows = colsum_partial_rows(dtype, T, N);
  if ((size_t)rows * (size_t)N > kStaticFloats) return BAMBOO_E_ARG;
  float* partial = nullptr;
  const int rc = scratch_for_current_device(&partial);
  if (rc != BAMBOO_OK) return rc;
  (void)hipGetLastError();
  // Every partial row that the final sum reads is written by the first kernel of this same call, so
  // nothing has to be cleared between calls; two calls that overlap on one GPU would race on the rows.
  const hipError_t e = launch_colsum_acc((hipStream_t)stream, dtype, T, N, A, out, partial);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return BAMBOO_E_HIP;
  }
  return BAMBOO_OK;
}

}  // extern "C"
