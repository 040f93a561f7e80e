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
// Workgroup g ranks the rows [g, g + 1) * kScan * kScanBatch.  It does not wait for the workgroups before it:
// it counts the kept rows ahead of its share itself (loads only, requested kScanBatch chunks at a time; at most
// a few shares, all L2 hits after the first reader), so no workgroup depends on another and the launch needs no
// counter that must start at zero.  The workgroup whose share holds the last active row writes *count.
static __global__ __launch_bounds__(kScan) void compact_rows_kernel(const int32_t* __restrict__ krow,
                                                                    int32_t* __restrict__ rowidx,
                                                                    int32_t* __restrict__ count,
                                                                    const int32_t* active,
                                                                    int rows_per_chain, int R, int T) {
  constexpr int NW = kScan / 64;
  constexpr int kShare = kScan * kScanBatch;
  __shared__ int wave_tot[kScanBatch][NW];
  __shared__ int wave_pre[NW];
  const int Ract = sdi::active_rows(active, rows_per_chain, R);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int start = static_cast<int>(blockIdx.x) * kShare;
  const int last_share = Ract > 0 ? (Ract - 1) / kShare : 0;
  if (static_cast<int>(blockIdx.x) > last_share) return;          // uniform over the workgroup

  // kept rows in the shares before this one (all of them lie below Ract)
  int mine = 0;
  for (int s0 = 0; s0 < start; s0 += kShare) {
    int k[kScanBatch];
#pragma unroll
    for (int c = 0; c < kScanBatch; ++c) k[c] = krow[s0 + c * kScan + tid];
#pragma unroll
    for (int c = 0; c < kScanBatch; ++c) mine += static_cast<unsigned>(k[c]) < static_cast<unsigned>(T) ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  if (lane == 0) wave_pre[wave] = mine;

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
  int base = 0;                                    // kept rows before the chunk (the same in every thread)
#pragma unroll
  for (int w = 0; w < NW; ++w) base += wave_pre[w];
#pragma unroll
  for (int c = 0; c < kScanBatch; ++c) {
    int before = 0, total = 0;                     // kept rows of chunk c in earlier wavefronts / in all
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int v = wave_tot[c][w];
      before += w < wave ? v : 0;
      total += v;
    }
    if (keep[c]) rowidx[base + before + __popcll(m[c] & ((1ull << lane) - 1ull))] = start + c * kScan + tid;
    base += total;
  }
  if (tid == 0 && static_cast<int>(blockIdx.x) == last_share) *count = base;
}

// workgroups compact_rows_kernel is launched with for R rows
static inline unsigned compact_rows_grid(int R) {
  const int share = kScan * kScanBatch;
  return static_cast<unsigned>(R > 0 ? (R + share - 1) / share : 1);
}

}  // namespace sdrows
