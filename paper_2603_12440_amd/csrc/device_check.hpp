// Host-side check shared by the entry points: is the current device a gfx950 GPU?
// Cached per device ordinal after the first query.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>

#include "../../include/gemm.h"

namespace mi355gemm {

inline std::atomic<int> g_dev_ok[64];   // 0 unknown, 1 ok, -1 not gfx950

inline int check_device_gfx950() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return GEMM_ERR_NO_DEVICE; }
  if (dev >= 64) return GEMM_ERR_NO_DEVICE;
  int st = g_dev_ok[dev].load(std::memory_order_acquire);
  if (st == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return GEMM_ERR_NO_DEVICE; }
    st = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
    g_dev_ok[dev].store(st, std::memory_order_release);
  }
  return st == 1 ? GEMM_OK : GEMM_ERR_NO_DEVICE;
}

}  // namespace mi355gemm
