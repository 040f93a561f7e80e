// Base of the target-prediction objects behind sdden.h.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>

#include "../../include/sdden.h"
#include "sd_internal.h"

struct sdden {
  virtual ~sdden() {}
  // Enqueue out[r] = D(X[r], krow[r]) for rows r < R with krow[r] >= 0.
  virtual int eval(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) = 0;
  // Allocate whatever per-call scratch evaluations of up to R rows need (setup time only).
  virtual int reserve(int R) { (void)R; return SD_OK; }
  int d = 0, T = 0;
  const int32_t* active = nullptr;   // optional device-side chain count
  int rows_per_chain = 1;
  std::string err;
};

namespace sdi {
extern std::string g_den_create_error;

// Rows to evaluate given the optional device-side chain count.
__device__ __forceinline__ int active_rows(const int32_t* active, int rows_per_chain, int R) {
  if (active == nullptr) return R;
  const long long lim = static_cast<long long>(*active) * rows_per_chain;
  return lim < R ? (lim < 0 ? 0 : static_cast<int>(lim)) : R;
}
}  // namespace sdi
