// Row bookkeeping shared by the GEMM-based denoisers: the rows of a batched target call that
// carry a chain step (krow >= 0) are gathered into a dense index list, so the GEMMs only spend
// MFMA work on rows that are really evaluated (the last draft of every chain and the rows past
// the end of a chain are masked).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "sdden_internal.h"

namespace sdrows {

constexpr int kScan = 1024;

// rowidx[0..count) = indices r < Ract with krow[r] >= 0, in increasing order; *count = how many.
static __global__ __launch_bounds__(kScan) void compact_rows_kernel(const int32_t* __restrict__ krow,
                                                                    int32_t* __restrict__ rowidx,
                                                                    int32_t* __restrict__ count,
                                                                    const int32_t* active,
                                                                    int rows_per_chain, int R) {
  __shared__ int wave_tot[kScan / 64];
  __shared__ int sh_base;
  const int Ract = sdi::active_rows(active, rows_per_chain, R);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) sh_base = 0;
  __syncthreads();
  for (int start = 0; start < Ract; start += kScan) {
    const int r = start + tid;
    const bool keep = r < Ract && krow[r] >= 0;
    const unsigned long long m = __ballot(keep);
    if (lane == 0) wave_tot[wave] = __popcll(m);
    __syncthreads();
    int offset = sh_base;
    for (int w = 0; w < wave; ++w) offset += wave_tot[w];
    if (keep) rowidx[offset + __popcll(m & ((1ull << lane) - 1ull))] = r;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < kScan / 64; ++w) tot += wave_tot[w];
      sh_base += tot;
    }
    __syncthreads();
  }
  if (tid == 0) *count = sh_base;
}

}  // namespace sdrows
