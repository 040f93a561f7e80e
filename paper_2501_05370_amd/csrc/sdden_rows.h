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

constexpr int kScanBatch = 8;      // chunks of kScan rows whose steps are requested together

// rowidx[0..count) = indices r < Ract with 0 <= krow[r] < T, in increasing order; *count = how many (a step
// index the chain does not have is a masked row like a negative one: the per-step tables end at T).
// One workgroup walks the rows; it is a chain of global-load round trips unless the loads are batched, so a
// thread requests its rows of kScanBatch chunks at once and the chunks are then ranked from registers.
static __global__ __launch_bounds__(kScan) void compact_rows_kernel(const int32_t* __restrict__ krow,
                                                                    int32_t* __restrict__ rowidx,
                                                                    int32_t* __restrict__ count,
                                                                    const int32_t* active,
                                                                    int rows_per_chain, int R, int T) {
  constexpr int NW = kScan / 64;
  __shared__ int wave_tot[kScanBatch][NW];
  const int Ract = sdi::active_rows(active, rows_per_chain, R);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int base = 0;                                    // kept rows before this batch (the same in every thread)
  for (int start = 0; start < Ract; start += kScan * kScanBatch) {
    bool keep[kScanBatch];
#pragma unroll
    for (int c = 0; c < kScanBatch; ++c) {
      const int r = start + c * kScan + tid;
      keep[c] = r < Ract && static_cast<unsigned>(krow[r]) < static_cast<unsigned>(T);
    }
    unsigned long long m[kScanBatch];
#pragma unroll
    for (int c = 0; c < kScanBatch; ++c) {
      m[c] = __ballot(keep[c]);
      if (lane == 0) wave_tot[c][wave] = __popcll(m[c]);
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kScanBatch; ++c) {
      int before = 0, total = 0;                   // kept rows of chunk c in earlier wavefronts / in all
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int v = wave_tot[c][w];
        before += w < wave ? v : 0;
        total += v;
      }
      if (keep[c]) rowidx[base + before + __popcll(m[c] & ((1ull << lane) - 1ull))] = start + c * kScan + tid;
      base += total;
    }
    __syncthreads();                               // wave_tot is rewritten by the next batch
  }
  if (tid == 0) *count = base;
}

}  // namespace sdrows
