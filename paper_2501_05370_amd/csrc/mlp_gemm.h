// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores with fused bias / SiLU epilogues, used by the
// MLP denoiser:  C[M,N] = A[M,K] * Bt[N,K]^T, both operands K-contiguous.
//
// Workgroup tile BM x BN x 64, WM x WN wavefronts, each wavefront owns (BM/WM) x (BN/WN) of the
// tile as 32x32 v_mfma_f32_32x32x16_bf16 accumulators.  The K-slice of both operands is staged in
// LDS (rows padded to 72 elements: the 16-byte fragment reads of any 8 consecutive lanes then cover
// all 32 banks); the next slice is fetched into registers while the current one feeds the MFMAs.
// A must be readable for all rows of every launched tile (callers round their row capacity up to a
// multiple of BM); rows >= M are computed on whatever is there and never stored.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace mlpgemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr int LDSK = BK + 8;      // padded LDS row, in bf16 elements
constexpr int kRowPad = 256;      // row capacity of A operands must be a multiple of this

struct Args {
  const uint16_t* A;     // [>= tiles*BM, Kdim] bf16, dense
  const uint16_t* Bt;    // [N, Kdim] bf16 (weights, transposed: row = output feature)
  int N, Kdim;
  const int32_t* count;  // device: M
  const int32_t* rowidx; // dense row -> source row
  const int32_t* krow;   // source row -> chain step
  const float* bias;     // EPI 1: per-step table [T, N]; EPI 2, 3: [N]
  uint16_t* outb;        // EPI 1, 2: bf16 [M, N] dense
  float* outf;           // EPI 3: fp32 [*, N] at source rows
};

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

__device__ __forceinline__ uint16_t to_bf16_bits(float x) {
  const __bf16 b = static_cast<__bf16>(x);
  uint16_t u;
  __builtin_memcpy(&u, &b, 2);
  return u;
}

template <int BM, int BN, int WM, int WN>
constexpr size_t lds_bytes() {
  return 2 * static_cast<size_t>(BM + BN) * LDSK * sizeof(uint16_t);
}

// EPI 1: out = bf16(silu(acc + bias[krow[src]][n]));  EPI 2: out = bf16(silu(acc + bias[n]));
// EPI 3: outf[src][n] = acc + bias[n].
template <int BM, int BN, int WM, int WN, int EPI, int PM = 4, int PN = 8>
__global__ __launch_bounds__(64 * WM * WN) void kernel(Args p) {
  constexpr int NT = 64 * WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;       // MFMA tiles per wavefront
  constexpr int ACH = BM * (BK / 8) / NT;                    // 16-byte chunks per thread per K-slice
  constexpr int BCH = BN * (BK / 8) / NT;
  constexpr int ROWS_PER_PASS = NT / 8;                      // tile rows covered by one chunk pass
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wavefront tile must be whole MFMA tiles");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "chunks must divide evenly");
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem);          // [2][BM][LDSK]
  uint16_t* Bs = As + 2 * BM * LDSK;                         // [2][BN][LDSK]

  const int M = *p.count;
  const int tiles_n = p.N / BN;
  // Workgroups are handed to the 8 XCDs round-robin (id % 8), and each XCD has its own L2.  Give
  // every XCD a contiguous run of tiles, ordered as PM x PN patches, so that the ~32 tiles an XCD
  // works on at a time share PM row panels of A and PN row panels of the weights.
  int tile_m, tile_n;
  {
    const int per_xcd = gridDim.x / 8;                           // host launches a multiple of 8
    const int L = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const int patches_n = (tiles_n + PN - 1) / PN;
    const int patch = L / (PM * PN), within = L % (PM * PN);
    tile_m = (patch / patches_n) * PM + within % PM;
    tile_n = (patch % patches_n) * PN + within / PM;
    if (tile_n >= tiles_n) return;
  }
  if (tile_m * BM >= M) return;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int half = lane >> 5, l32 = lane & 31;
  const int Kd = p.Kdim;

  // this thread's 16-byte chunk: tile row t/8 (+ ROWS_PER_PASS per pass), K offset 8*(t%8)
#ifdef MLPGEMM_EXPERIMENT_SAME_PANEL   /* measurement experiment only: every tile reads panel 0 */
  const uint16_t* a_thr = p.A + (static_cast<size_t>(0) * BM + (t >> 3)) * Kd + 8 * (t & 7);
  const uint16_t* b_thr = p.Bt + (static_cast<size_t>(0) * BN + (t >> 3)) * Kd + 8 * (t & 7);
#else
  const uint16_t* a_thr = p.A + (static_cast<size_t>(tile_m) * BM + (t >> 3)) * Kd + 8 * (t & 7);
  const uint16_t* b_thr = p.Bt + (static_cast<size_t>(tile_n) * BN + (t >> 3)) * Kd + 8 * (t & 7);
#endif
  const int lds_thr = (t >> 3) * LDSK + 8 * (t & 7);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  u32x4 ra[ACH], rb[BCH];
#define MLPGEMM_FETCH(k0)                                                                              \
  do {                                                                                                 \
    _Pragma("unroll") for (int i_ = 0; i_ < ACH; ++i_)                                                 \
        ra[i_] = *reinterpret_cast<const u32x4*>(a_thr + static_cast<size_t>(i_) * ROWS_PER_PASS * Kd + (k0)); \
    _Pragma("unroll") for (int i_ = 0; i_ < BCH; ++i_)                                                 \
        rb[i_] = *reinterpret_cast<const u32x4*>(b_thr + static_cast<size_t>(i_) * ROWS_PER_PASS * Kd + (k0)); \
  } while (0)
#define MLPGEMM_STASH(s_)                                                                              \
  do {                                                                                                 \
    _Pragma("unroll") for (int i_ = 0; i_ < ACH; ++i_)                                                 \
        *reinterpret_cast<u32x4*>(As + (s_) * BM * LDSK + lds_thr + i_ * ROWS_PER_PASS * LDSK) = ra[i_]; \
    _Pragma("unroll") for (int i_ = 0; i_ < BCH; ++i_)                                                 \
        *reinterpret_cast<u32x4*>(Bs + (s_) * BN * LDSK + lds_thr + i_ * ROWS_PER_PASS * LDSK) = rb[i_]; \
  } while (0)

  const int nk = Kd / BK;
  MLPGEMM_FETCH(0);
  MLPGEMM_STASH(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int s = kt & 1;
    if (kt + 1 < nk) MLPGEMM_FETCH((kt + 1) * BK);
    const uint16_t* Aw = As + s * BM * LDSK + (wm * (BM / WM) + l32) * LDSK + 8 * half;
    const uint16_t* Bw = Bs + s * BN * LDSK + (wn * (BN / WN) + l32) * LDSK + 8 * half;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Aw + i * 32 * LDSK + kk));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bw + j * 32 * LDSK + kk));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) MLPGEMM_STASH(s ^ 1);
    __syncthreads();
  }
#undef MLPGEMM_FETCH
#undef MLPGEMM_STASH

  // ---- epilogue: element (row = (v/4)*8 + half*4 + v%4, col = l32) of each 32x32 tile
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gm = tile_m * BM + wm * (BM / WM) + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
      if (gm >= M) continue;
      const int src = p.rowidx[gm];
      const float* brow = EPI == 1 ? p.bias + static_cast<size_t>(p.krow[src]) * p.N : p.bias;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int gn = tile_n * BN + wn * (BN / WN) + j * 32 + l32;
        const float c = acc[i][j][v] + brow[gn];
        if (EPI == 3) p.outf[static_cast<size_t>(src) * p.N + gn] = c;
        else p.outb[static_cast<size_t>(gm) * p.N + gn] = to_bf16_bits(silu(c));
      }
    }
  }
}

// Enqueue the GEMM for up to Rmax rows (the kernel reads the true M on the device).
template <int BM, int BN, int WM, int WN, int EPI, int PM = 4, int PN = 8>
hipError_t launch(const Args& a, int Rmax, hipStream_t st) {
  constexpr size_t shmem = lds_bytes<BM, BN, WM, WN>();
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel<BM, BN, WM, WN, EPI, PM, PN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (Rmax + BM - 1) / BM, tiles_n = a.N / BN;
  const int patches = ((tiles_m + PM - 1) / PM) * ((tiles_n + PN - 1) / PN);
  const int grid = (patches * PM * PN + 7) / 8 * 8;
  hipLaunchKernelGGL((kernel<BM, BN, WM, WN, EPI, PM, PN>), dim3(grid), dim3(64 * WM * WN), shmem, st, a);
  return hipGetLastError();
}

}  // namespace mlpgemm
