// fp32 x fp32 -> fp32 GEMM on the gfx950 matrix cores for the two skinny products of the low-rank
// Gaussian denoiser:  C[M,N] = A[M,K] * Bt[N,K]^T, both operands K-contiguous, rows of A optionally
// gathered through an index.
//
// Same skeleton as the bf16 MLP GEMM: BM x BN x 32 workgroup tile, WM x WN wavefronts of 32x32
// v_mfma_f32_32x32x2f32 accumulators, K-slices of 32 floats (128 B per row) loaded from global memory
// straight into LDS (a wavefront load fills 8 rows, lane l landing at byte 16*l, the lane fetching
// chunk (l%8) ^ ((row >> 1) & 7) of its row so that fragment reads are bank-conflict free on the 64-bank
// LDS: see the bf16 GEMM), an NS-stage LDS
// ring with a workgroup barrier that leaves loads in flight.
// Fragments: a lane reads one 16-byte chunk = 4 consecutive k of its row and feeds 4 MFMAs; the two
// lane halves of an MFMA (k index 0 / 1 of the instruction) read chunks 2m / 2m+1, i.e. MFMA e of
// step m contracts k = 8m+e and k = 8m+4+e.  Both operands use the same pairing, so the sum over the
// slice is the plain dot product.
// An MFMA of this shape runs 64 cycles for 4096 flop, so LDS and global traffic are far from
// binding; what matters is that every SIMD always has a wavefront with MFMAs to issue.  The first
// product (N = rank, long K) has few output tiles: its K range is split over gridDim.y and the
// partial sums go to separate slabs that a second small kernel adds in a fixed order (no atomics:
// results do not depend on scheduling).
// The Bt fragment is the FIRST MFMA operand: the accumulator tile is then C^T, a lane owns one row m of C and,
// per 32x32 tile, four runs of 4 consecutive columns, so everything the epilogues move (partial slabs, the X
// tile, the output) goes as 16-byte accesses, 16 per thread instead of 64 four-byte ones.  The second product
// has K = rank: its K loop is as short as its prologue and epilogue, and those are what its speed hangs on.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lrgemm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 32;

struct __attribute__((aligned(16))) RowInfo {
  int32_t src;
  float gp, cf;
  int32_t pad;
};

struct Args {
  const float* A;          // rows of lda floats; tile row r reads row arow[r] (or r when arow is null)
  const int32_t* arow;
  int64_t lda;
  const float* Bt;         // [N, ldb]
  int64_t ldb;
  int N, Kdim;             // Kdim: the whole contraction length (multiple of 32 * gridDim.y)
  const int32_t* count;    // device: M
  // stage 1: partial sums, slab s = part + s * slab_stride, dense rows of N floats
  float* part;
  int64_t slab_stride;
  // stage 2 epilogue: out[src] = acc + gp X[src] + cf mu with (src, gp, cf) = rowinfo[gm], which
  // reduce_gain_kernel fills: src = rowidx[gm], gp = gperp[krow[src]], cf = coef[krow[src]]
  const RowInfo* rowinfo;
  const float* X;
  float* out;
  const float* mu;
};

template <int N>
__device__ __forceinline__ void wait_loads() {
  static_assert(N == 0 || N == 4 || N == 8 || N == 16, "add the count");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}

__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int BM, int BN, int WM, int WN, int STAGE, int NS>
__global__ __launch_bounds__(64 * WM * WN) void kernel(Args p) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int APASS = BM / 8 / NW, BPASS = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups must divide evenly");
  static_assert(NW % 2 == 0, "the chunk permutation takes the parity of a row group from the wavefront index");
  extern __shared__ __align__(1024) unsigned char smem[];
  unsigned char* As = smem;                                  // [NS][BM][128 B]
  unsigned char* Bs = smem + NS * BM * 128;                  // [NS][BN][128 B]

  const int M = *p.count;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  if (tile_m * BM >= M) return;
  const int nk = p.Kdim / BK / gridDim.y;                    // slices of this split
  const int64_t kbase = static_cast<int64_t>(blockIdx.y) * nk * BK * 4;   // byte offset of the split's first k

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int half = lane >> 5, l32 = lane & 31;
  const int lrow = lane >> 3, lchunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);   // (LDS row >> 1) & 7, see above

  // source rows of this lane's loads (rows past M / N are clamped: computed, never stored)
  const unsigned char* a_src[APASS];
  const unsigned char* b_src[BPASS];
#pragma unroll
  for (int i = 0; i < APASS; ++i) {
    int r = tile_m * BM + 8 * (i * NW + wave) + lrow;
    r = r < M ? r : M - 1;
    const int64_t row = p.arow ? p.arow[r] : r;
    a_src[i] = reinterpret_cast<const unsigned char*>(p.A + row * p.lda) + kbase + 16 * lchunk;
  }
#pragma unroll
  for (int i = 0; i < BPASS; ++i) {
    int r = tile_n * BN + 8 * (i * NW + wave) + lrow;
    r = r < p.N ? r : p.N - 1;
    b_src[i] = reinterpret_cast<const unsigned char*>(p.Bt + static_cast<int64_t>(r) * p.ldb) + kbase + 16 * lchunk;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  typedef __attribute__((address_space(3))) void* lds_ptr;
  typedef const __attribute__((address_space(1))) void* gbl_ptr;
#define LRGEMM_FETCH(s_, kt_)                                                                          \
  do {                                                                                                   \
    _Pragma("unroll") for (int i_ = 0; i_ < APASS; ++i_)                                                 \
        __builtin_amdgcn_global_load_lds((gbl_ptr)(a_src[i_] + (kt_) * (BK * 4)),                        \
                                         (lds_ptr)(As + (s_) * BM * 128 + (i_ * NW + wave) * 1024), 16, 0, 0); \
    _Pragma("unroll") for (int i_ = 0; i_ < BPASS; ++i_)                                                 \
        __builtin_amdgcn_global_load_lds((gbl_ptr)(b_src[i_] + (kt_) * (BK * 4)),                        \
                                         (lds_ptr)(Bs + (s_) * BN * 128 + (i_ * NW + wave) * 1024), 16, 0, 0); \
  } while (0)

#pragma unroll
  for (int k = 0; k < NS - 1; ++k)
    if (k < nk) LRGEMM_FETCH(k, k);

  // STAGE 2: everything the epilogue needs from memory is requested here, while the first slices are on
  // their way: a lane's two rows of the tile (source row and per-row scalars, one 16-byte record each), then
  // its 64 elements of X as 16 16-byte loads.  Left to the epilogue these are dependent round trips per row
  // group, as much as the short K loop (K = rank) itself.
  f32x4 xv[STAGE == 2 ? TM : 1][TN][4];
  f32x4 muv[STAGE == 2 ? TN : 1][4];
  int rsrc[TM];
  float rgp[TM], rcf[TM];
  if (STAGE == 2) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int gm = tile_m * BM + wm * (BM / WM) + i * 32 + l32;
      const RowInfo info = p.rowinfo[gm < M ? gm : M - 1];
      rsrc[i] = gm < M ? info.src : -1;
      rgp[i] = info.gp;
      rcf[i] = info.cf;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int gn = tile_n * BN + wn * (BN / WN) + j * 32 + q * 8 + half * 4;
        muv[j][q] = gn < p.N ? *reinterpret_cast<const f32x4*>(p.mu + gn) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < TM; ++i)
          xv[i][j][q] = (rsrc[i] >= 0 && gn < p.N)
                            ? *reinterpret_cast<const f32x4*>(p.X + static_cast<int64_t>(rsrc[i]) * p.N + gn)
                            : f32x4{0.f, 0.f, 0.f, 0.f};
      }
  }

  const int a_row = (wm * (BM / WM) + l32) * 128, b_row = (wn * (BN / WN) + l32) * 128;
  const int sw = (l32 >> 1) & 7;
  for (int kt = 0; kt < nk; ++kt) {
    const int s = kt % NS;
    if (kt + NS - 1 < nk) {
      wait_loads<(NS - 2) * (APASS + BPASS)>();
      barrier_keep_loads();
      LRGEMM_FETCH((kt + NS - 1) % NS, kt + NS - 1);
    } else {
      wait_loads<0>();
      barrier_keep_loads();
    }
    const unsigned char* Aw = As + s * BM * 128 + a_row;
    const unsigned char* Bw = Bs + s * BN * 128 + b_row;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int off = ((2 * m + half) ^ sw) << 4;
      f32x4 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = __builtin_bit_cast(f32x4, *reinterpret_cast<const u32x4*>(Aw + i * 32 * 128 + off));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = __builtin_bit_cast(f32x4, *reinterpret_cast<const u32x4*>(Bw + j * 32 * 128 + off));
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j][e], a[i][e], acc[i][j], 0, 0, 0);
    }
  }
#undef LRGEMM_FETCH

  // acc[i][j][4q + e] is element (row m = l32, column n = 8q + 4 half + e) of its 32x32 tile of C
  if (STAGE == 1) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int gm = tile_m * BM + wm * (BM / WM) + i * 32 + l32;
      if (gm >= M) continue;
      float* dst = p.part + static_cast<int64_t>(blockIdx.y) * p.slab_stride + static_cast<int64_t>(gm) * p.N;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gn = tile_n * BN + wn * (BN / WN) + j * 32 + q * 8 + half * 4;
          if (gn < p.N)
            *reinterpret_cast<f32x4*>(dst + gn) =
                f32x4{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        }
    }
  }
  if (STAGE == 2) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if (rsrc[i] < 0) continue;
      float* dst = p.out + static_cast<int64_t>(rsrc[i]) * p.N;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gn = tile_n * BN + wn * (BN / WN) + j * 32 + q * 8 + half * 4;
          if (gn >= p.N) continue;
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = acc[i][j][4 * q + e] + rgp[i] * xv[i][j][q][e] + rcf[i] * muv[j][q][e];
          *reinterpret_cast<f32x4*>(dst + gn) = o;
        }
    }
  }
}

// P'[gm][a] = gain[k][a] * (sum_s part_s[gm][a] - sab[k] qmu[a]),  k = krow[rowidx[gm]]; slabs added in order.
// Also leaves the per-row record of the second product's epilogue (source row, gperp[k], coef[k]).
__global__ __launch_bounds__(256) void reduce_gain_kernel(const float* __restrict__ part, int64_t slab_stride, int nsplit,
                                                          const int32_t* __restrict__ count, const int32_t* __restrict__ rowidx,
                                                          const int32_t* __restrict__ krow, const float* __restrict__ gain,
                                                          const float* __restrict__ sab, const float* __restrict__ qmu,
                                                          float* __restrict__ P, int N, const float* __restrict__ gperp,
                                                          const float* __restrict__ coef, RowInfo* __restrict__ rowinfo) {
  const int M = *count;
  const int n4 = N / 4;
  const int64_t g = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (g >= static_cast<int64_t>(M) * n4) return;
  const int gm = static_cast<int>(g / n4), c = static_cast<int>(g % n4) * 4;
  const int src = rowidx[gm];
  const int k = krow[src];
  if (c == 0) rowinfo[gm] = RowInfo{src, gperp[k], coef[k], 0};
  const int64_t o = static_cast<int64_t>(gm) * N + c;
  float4 s = *reinterpret_cast<const float4*>(part + o);
  for (int i = 1; i < nsplit; ++i) {
    const float4 v = *reinterpret_cast<const float4*>(part + i * slab_stride + o);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  const float4 gn = *reinterpret_cast<const float4*>(gain + static_cast<int64_t>(k) * N + c);
  const float4 q = *reinterpret_cast<const float4*>(qmu + c);
  const float sb = sab[k];
  float4 r;
  r.x = gn.x * (s.x - sb * q.x); r.y = gn.y * (s.y - sb * q.y);
  r.z = gn.z * (s.z - sb * q.z); r.w = gn.w * (s.w - sb * q.w);
  *reinterpret_cast<float4*>(P + o) = r;
}

// Raises the kernel's dynamic-LDS limit on the current device; done for every instantiation when a denoiser is
// created, never on the launch path (no one-time calls or "already done" flags between a caller and its launches:
// a HIP graph can capture the very first use).
template <int BM, int BN, int WM, int WN, int STAGE, int NS>
hipError_t prepare() {
  constexpr size_t shmem = NS * static_cast<size_t>(BM + BN) * 128;
  static_assert(NS >= 2 && shmem <= 160 * 1024, "ring must fit the 160 KiB of LDS");
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel<BM, BN, WM, WN, STAGE, NS>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
}

template <int BM, int BN, int WM, int WN, int STAGE, int NS>
hipError_t launch(const Args& a, int Rmax, int nsplit, hipStream_t st) {
  constexpr size_t shmem = NS * static_cast<size_t>(BM + BN) * 128;
  const int tiles = ((Rmax + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL((kernel<BM, BN, WM, WN, STAGE, NS>), dim3(tiles, nsplit), dim3(64 * WM * WN), shmem, st, a);
  return hipGetLastError();
}

}  // namespace lrgemm
