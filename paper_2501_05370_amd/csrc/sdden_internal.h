// Base of the target-prediction objects behind sdden.h.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sdden.h"
#include "sd_internal.h"

// HIP-event timing of one chosen kernel inside sdden_eval (measurement only; off by default).
struct sdden_profiler {
  int which = 0;                       // 0 = off, else the 1-based index of the timed kernel
  int min_rows = 0, cur_rows = 0;      // only calls with at least min_rows rows are timed
  std::vector<hipEvent_t> events;      // start/stop pairs, reused between collections
  size_t used = 0;
  ~sdden_profiler() {
    for (hipEvent_t e : events) (void)hipEventDestroy(e);
  }
  void mark(int kernel_index, hipStream_t st) {
    if (which != kernel_index || cur_rows < min_rows) return;
    if (used == events.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return;
      events.push_back(e);
    }
    (void)hipEventRecord(events[used++], st);
  }
};

struct sdden {
  virtual ~sdden() {}
  // Enqueue out[r] = D(X[r], krow[r]) for rows r < R with krow[r] >= 0.
  virtual int eval(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) = 0;
  // Allocate whatever per-call scratch evaluations of up to R rows need (setup time only).
  virtual int reserve(int R) { (void)R; return SD_OK; }
  // X with a caller-provided bf16 image of the same rows; denoisers without a use for it ignore it
  virtual int eval_mirror(int R, const float* X, const uint16_t* Xbf16, const int32_t* krow, float* out, hipStream_t st) {
    (void)Xbf16;
    return eval(R, X, krow, out, st);
  }
  int d = 0, T = 0;
  sdden_profiler prof;
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
