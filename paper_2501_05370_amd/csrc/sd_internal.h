// Shared host-side plumbing of the library: error text, HIP call checking, context layout.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>

#include "../../include/sd.h"

struct sd_ctx {
  int32_t T = 0, d = 0, K = 0;
  uint64_t seed = 0;
  int mode = SD_DRAFT_FROZEN;
  double tau = 1.0;
  int verify_shape = 0;         // 0 = default launch shape of the verify kernel, else a measured alternative
  float* dev_a = nullptr;       // [T] each, one allocation of 3T floats
  float* dev_c = nullptr;
  float* dev_sigma = nullptr;
  int32_t* dev_queue = nullptr;  // counter behind the schedule: chain dispenser of the Langevin wavefront kernel
  int cus = 256;                 // compute units of the context's device
  const int32_t* active = nullptr;
  const float* carry_src = nullptr;    // FROZEN_REUSED: predictions [B,K+1,d] of the window just verified
  float* carry_dst = nullptr;          //   and the [B,d] frozen predictions sd_advance fills for the next one
  int carry_rule = 0;                  // SD_CARRY_DRAFT / SD_CARRY_LAST_ACCEPTED
  uint16_t* draft_mirror = nullptr;    // optional bf16 image of the drafted rows, same layout as Ytilde
  const float* start_pred = nullptr;   // EXPLICIT mode: D(y_n, n) as [B,d], replaces row 0 of Dq
  void* ws = nullptr;
  size_t ws_bytes = 0;
  void* static_ws = nullptr;           // this device's copy of the library's static scratch (sd_advance_static)
  int device = 0;
  std::string err;
};

namespace sdi {

inline int fail(std::string& slot, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  slot = buf;
  return code;
}

#define SD_HIP_TRY(slot, expr)                                                          \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess)                                                               \
      return sdi::fail(slot, SD_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

hipError_t langevin_prepare(int* cus);   // sd_langevin.hip: kernel attributes + CU count, once per sd_create

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace sdi
