// bf16 x bf16 -> fp32 GEMM on the gfx950 matrix cores with fused bias / SiLU epilogues, used by the
// MLP denoiser:  C[M,N] = A[M,K] * Bt[N,K]^T, both operands K-contiguous.
//
// Workgroup tile BM x BN x 64, WM x WN wavefronts, each wavefront owns (BM/WM) x (BN/WN) of the
// tile as 32x32 v_mfma_f32_32x32x16_bf16 accumulators.  K-slices go from global memory straight
// into LDS (global_load_lds_dwordx4): no staging registers and no LDS store instructions.  One
// wavefront load fills 1 KiB of LDS = 8 rows of a 64-element slice, lane l landing at byte 16*l;
// bank conflicts are avoided by permuting which 16-byte chunk of its row a lane fetches
// (chunk ^ ((row >> 1) & 7), row = the row's place in the LDS tile) instead of padding rows.  The LDS of
// gfx950 serves a 128-bit read 16 lanes at a time out of 64 four-byte banks, so the 16-byte reads of 16
// consecutive rows at one k-chunk must fall on 16 different places modulo 256 bytes: two rows are 256
// bytes, so the row's parity picks the half and (row >> 1) & 7 has to run through all eight chunks.
// The permutation chunk ^ (row & 7), which is the one for 32 banks, reads at half the rate here
// (measured: 123 against 224 bytes per clock and CU, SQ_LDS_BANK_CONFLICT equal to the busy cycles).  NS LDS stages form a ring: up to NS-1 slices stream in while the
// current one feeds the MFMAs.  The per-slice workgroup barrier is a bare s_barrier behind
// s_waitcnt vmcnt(n): __syncthreads() would drain every outstanding load and empty the ring.
// The 256 x 256 tile fills LDS with two stages; the 128 x 128 tile used for few rows runs four,
// which hides the load latency that otherwise bounds it (one workgroup per CU, half the CUs).
// Tiles are ordered in PM x PN patches per XCD (workgroups go to the 8 XCDs round-robin and
// each XCD has its own L2).
// A must be readable for all rows of every launched tile (callers round their row capacity up to
// kRowPad); rows >= M are computed on whatever is there and never stored.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace mlpgemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr int kRowPad = 256;      // row capacity of A operands must be a multiple of this

struct Args {
  const uint16_t* A;     // [>= tiles*BM, Kdim] bf16, dense; or, with arow, the rows arow[m] of a larger matrix
  const int32_t* arow;   // optional gather index for the rows of A (dense row m reads A[arow[m]])
  const uint16_t* Bt;    // [N, Kdim] bf16 (weights, transposed: row = output feature)
  int N, Kdim;
  const int32_t* count;  // device: M
  const int32_t* rowidx; // dense row -> source row
  const int32_t* krow;   // source row -> chain step
  const float* bias;     // EPI 1: per-step table [T, N]; EPI 2, 3: [N]
  uint16_t* outb;        // EPI 1, 2: bf16 [M, N] dense
  float* outf;           // EPI 3: fp32 [*, N] at source rows
};

// x * sigmoid(x) with the hardware reciprocal (1 ulp): the quotient form compiles to the ten-instruction
// correctly rounded division, for a result that is rounded to bf16 next.
__device__ __forceinline__ float silu(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

__device__ __forceinline__ uint16_t to_bf16_bits(float x) {
  const __bf16 b = static_cast<__bf16>(x);
  uint16_t u;
  __builtin_memcpy(&u, &b, 2);
  return u;
}

// waits until at most N of this wavefront's vector-memory loads are outstanding (they complete in order)
template <int N>
__device__ __forceinline__ void wait_loads() {
  static_assert(N == 0 || N == 4 || N == 6 || N == 8 || N == 12 || N == 16 || N == 24, "add the count");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if constexpr (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
  if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if constexpr (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
  if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  if constexpr (N == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
}

// workgroup barrier that leaves vector-memory loads in flight (LDS traffic of this wavefront is drained)
__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// EPI 1: out = bf16(silu(acc + bias[krow[src]][n]));  EPI 2: out = bf16(silu(acc + bias[n]));
// EPI 3: outf[src][n] = acc + bias[n].
template <int BM, int BN, int WM, int WN, int EPI, int NS, bool GATHER = false, int PM = 4, int PN = 8>
__global__ __launch_bounds__(64 * WM * WN) void kernel(Args p) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int APASS = BM / 8 / NW, BPASS = BN / 8 / NW;    // wavefront loads per K-slice
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "row groups must divide evenly");
  static_assert(NW % 2 == 0, "the chunk permutation takes the parity of a row group from the wavefront index");
  extern __shared__ __align__(1024) unsigned char smem[];
  unsigned char* As = smem;                                  // [NS][BM][128 B]
  unsigned char* Bs = smem + NS * BM * 128;                  // [NS][BN][128 B]

  const int M = *p.count;
  const int tiles_n = p.N / BN;
  int tile_m, tile_n;
  {
    const int per_xcd = gridDim.x / 8;
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

  // lane's source: row (8*group + lane/8), 16-byte chunk (lane%8) ^ ((row >> 1) & 7); the group's parity is the wavefront's
  const int lrow = lane >> 3, lchunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);   // (LDS row >> 1) & 7, see above
  const unsigned char* a_lane = reinterpret_cast<const unsigned char*>(p.A) +
                                (static_cast<size_t>(tile_m) * BM + 8 * wave + lrow) * Kd * 2 + 16 * lchunk;
  const unsigned char* b_lane = reinterpret_cast<const unsigned char*>(p.Bt) +
                                (static_cast<size_t>(tile_n) * BN + 8 * wave + lrow) * Kd * 2 + 16 * lchunk;
  const size_t pass_stride = static_cast<size_t>(8 * NW) * Kd * 2;
  // gathered A: one source row per load pass (rows past M repeat the last one: computed, never stored)
  const unsigned char* a_src[GATHER ? APASS : 1];
  if (GATHER) {
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
      int r = tile_m * BM + 8 * (i * NW + wave) + lrow;
      r = r < M ? r : M - 1;
      a_src[i] = reinterpret_cast<const unsigned char*>(p.A) + static_cast<size_t>(p.arow[r]) * Kd * 2 + 16 * lchunk;
    }
  }

  // the epilogue's row bookkeeping is fetched now, one row per thread, and parked in LDS (see kernel_hs)
  static_assert(BM <= 64 * WM * WN, "one thread per tile row");
  __shared__ int sh_src[BM], sh_step[BM];
  if (t < BM) {
    const int gm = tile_m * BM + t;
    const int src = p.rowidx[gm < M ? gm : M - 1];
    sh_src[t] = src;
    sh_step[t] = EPI == 1 ? p.krow[src] : 0;
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
#define MLPGEMM_FETCH(s_, k0)                                                                        \
  do {                                                                                                 \
    _Pragma("unroll") for (int i_ = 0; i_ < APASS; ++i_)                                               \
        __builtin_amdgcn_global_load_lds((gbl_ptr)((GATHER ? a_src[GATHER ? i_ : 0] : a_lane + i_ * pass_stride) + (k0) * 2), \
                                         (lds_ptr)(As + (s_) * BM * 128 + (i_ * NW + wave) * 1024), 16, 0, 0); \
    _Pragma("unroll") for (int i_ = 0; i_ < BPASS; ++i_)                                               \
        __builtin_amdgcn_global_load_lds((gbl_ptr)(b_lane + i_ * pass_stride + (k0) * 2),              \
                                         (lds_ptr)(Bs + (s_) * BN * 128 + (i_ * NW + wave) * 1024), 16, 0, 0); \
  } while (0)

  const int nk = Kd / BK;
#pragma unroll
  for (int k = 0; k < NS - 1; ++k)
    if (k < nk) MLPGEMM_FETCH(k, k * BK);
  // fragment addressing: row r, chunk c -> r*128 + ((c ^ ((r >> 1) & 7)) << 4); tiles start at multiples of 32 rows
  const int a_row = (wm * (BM / WM) + l32) * 128, b_row = (wn * (BN / WN) + l32) * 128;
  const int sw = (l32 >> 1) & 7;
  for (int kt = 0; kt < nk; ++kt) {
    const int s = kt % NS;
    // slice kt has landed once only the NS-2 younger slices are outstanding; past the barrier every
    // wavefront is done with slice kt-1, whose stage takes slice kt+NS-1
    if (kt + NS - 1 < nk) {
      wait_loads<(NS - 2) * (APASS + BPASS)>();
      barrier_keep_loads();
      MLPGEMM_FETCH((kt + NS - 1) % NS, (kt + NS - 1) * BK);
    } else {
      wait_loads<0>();
      barrier_keep_loads();
    }
    const unsigned char* Aw = As + s * BM * 128 + a_row;
    const unsigned char* Bw = Bs + s * BN * 128 + b_row;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int off = ((2 * kk + half) ^ sw) << 4;
      bf16x8 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Aw + i * 32 * 128 + off));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bw + j * 32 * 128 + off));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
#undef MLPGEMM_FETCH

  // EPI 2, 3: the bias depends on the column only and is read once, ahead of the stores (the fp32
  // stores of EPI 3 could alias it as far as the compiler knows, which would put a load behind each)
  float bcol[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bcol[j] = EPI == 1 ? 0.f : p.bias[tile_n * BN + wn * (BN / WN) + j * 32 + l32];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int lm = wm * (BM / WM) + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
      const int gm = tile_m * BM + lm;
      if (gm >= M) continue;
      const int src = sh_src[lm];
      const float* brow = EPI == 1 ? p.bias + static_cast<size_t>(sh_step[lm]) * p.N : p.bias;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int gn = tile_n * BN + wn * (BN / WN) + j * 32 + l32;
        const float c = acc[i][j][v] + (EPI == 1 ? brow[gn] : bcol[j]);
        if (EPI == 3) p.outf[static_cast<size_t>(src) * p.N + gn] = c;
        else p.outb[static_cast<size_t>(gm) * p.N + gn] = to_bf16_bits(silu(c));
      }
    }
  }
}

// Raises the kernel's dynamic-LDS limit on the current device.  Done for every instantiation when a denoiser is
// created, never on the launch path: the launch sequence is then free of one-time set-up calls (a HIP graph can
// capture its very first use) and of unsynchronised "already done" flags.
template <int BM, int BN, int WM, int WN, int EPI, int NS, bool GATHER = false, int PM = 4, int PN = 8>
hipError_t prepare() {
  constexpr size_t shmem = NS * static_cast<size_t>(BM + BN) * 128;
  static_assert(NS >= 2 && shmem <= 160 * 1024, "ring must fit the 160 KiB of LDS");
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel<BM, BN, WM, WN, EPI, NS, GATHER, PM, PN>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem));
}

// prepare<...>() must have run for the instantiation on this device.
template <int BM, int BN, int WM, int WN, int EPI, int NS, bool GATHER = false, int PM = 4, int PN = 8>
hipError_t launch(const Args& a, int Rmax, hipStream_t st) {
  constexpr size_t shmem = NS * static_cast<size_t>(BM + BN) * 128;
  const int tiles_m = (Rmax + BM - 1) / BM, tiles_n = a.N / BN;
  const int patches = ((tiles_m + PM - 1) / PM) * ((tiles_n + PN - 1) / PN);
  const int grid = (patches * PM * PN + 7) / 8 * 8;
  hipLaunchKernelGGL((kernel<BM, BN, WM, WN, EPI, NS, GATHER, PM, PN>), dim3(grid), dim3(64 * WM * WN), shmem, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Hand-scheduled form of the 256 x 256 x 64 tile (8 wavefronts 2 x 4, two LDS stages), used when the
// contraction has an even number (>= 2) of 64-wide slices.  Same operands, LDS layout and epilogues
// as the generic kernel above.  What differs is who places the waits:
//  * fragment reads are inline-asm ds_read_b128 and every s_waitcnt lgkmcnt(n) is written by hand, the
//    fragments it releases being operands of the wait so that no MFMA can move above it.  The compiler
//    left to itself waits for lgkmcnt(0) at every k-step (it loses count across the loop back-edge and
//    across inline asm), which exposes the LDS latency four times per slice;
//  * two fragment sets alternate per 16-wide k-step: the reads of step k+1 are issued before the
//    MFMAs of step k;
//  * the workgroup barrier sits before the MFMAs of the slice's last k-step (all fragment reads of
//    the stage have returned by then), so those MFMAs cover the issue of the next global loads and
//    the first fragment reads of the next slice.
// A hazard of this style: to the compiler an inline-asm read has completed when the statement ends, so it
// is free to copy a fragment register (a PHI at the loop's back-edge, a merge after a branch) while the
// data is still on its way.  The loop below carries its fragments in the registers the reads wrote (no
// branch between a read and its wait; checked in the generated code: no move of a fragment register);
// after a change of the loop structure or of the compiler the parity tests of the MLP denoiser are the
// check -- a copied in-flight register shows up as errors of order one, not of rounding size.
// ---------------------------------------------------------------------------------------------
template <int EPI, bool GATHER = false, int PM = 4, int PN = 8>
__global__ __launch_bounds__(512) void kernel_hs(Args p) {
  constexpr int BM = 256, BN = 256, WN = 4, NW = 8, TM = 4, TN = 2, APASS = 4, BPASS = 4;
  extern __shared__ __align__(1024) unsigned char smem[];
  const int M = *p.count;
  const int tiles_n = p.N / BN;
  int tile_m, tile_n;
  {
    const int per_xcd = gridDim.x / 8;
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
  const int lrow = lane >> 3, lchunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);   // (LDS row >> 1) & 7, see above
  const unsigned char* b_lane = reinterpret_cast<const unsigned char*>(p.Bt) +
                                (static_cast<size_t>(tile_n) * BN + 8 * wave + lrow) * Kd * 2 + 16 * lchunk;
  const size_t pass_stride = static_cast<size_t>(8 * NW) * Kd * 2;
  const unsigned char* a_src[APASS];
#pragma unroll
  for (int i = 0; i < APASS; ++i) {
    int r = tile_m * BM + 8 * (i * NW + wave) + lrow;
    if (GATHER) r = p.arow[r < M ? r : M - 1];
    a_src[i] = reinterpret_cast<const unsigned char*>(p.A) + static_cast<size_t>(r) * Kd * 2 + 16 * lchunk;
  }

  // the epilogue's row bookkeeping (dense row -> source row -> chain step) is fetched now, one row per thread,
  // and parked in LDS: after the K loop it would be two dependent round trips ahead of the bias loads, with
  // nothing else on the CU to hide them (the barriers of the K loop order these writes before the reads)
  __shared__ int sh_src[BM], sh_step[BM];
  if (t < BM) {
    const int gm = tile_m * BM + t;
    const int src = p.rowidx[gm < M ? gm : M - 1];
    sh_src[t] = src;
    sh_step[t] = EPI == 1 ? p.krow[src] : 0;
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
  // LDS map: A stage s at s * 32 KiB, B stage s at 64 KiB + s * 32 KiB
#define MLPHS_FETCH(s_, k0)                                                                            \
  do {                                                                                                   \
    _Pragma("unroll") for (int i_ = 0; i_ < APASS; ++i_)                                                 \
        __builtin_amdgcn_global_load_lds((gbl_ptr)(a_src[i_] + (k0) * 2),                                \
                                         (lds_ptr)(smem + (s_) * 32768 + (i_ * NW + wave) * 1024), 16, 0, 0); \
    _Pragma("unroll") for (int i_ = 0; i_ < BPASS; ++i_)                                                 \
        __builtin_amdgcn_global_load_lds((gbl_ptr)(b_lane + i_ * pass_stride + (k0) * 2),                \
                                         (lds_ptr)(smem + 65536 + (s_) * 32768 + (i_ * NW + wave) * 1024), 16, 0, 0); \
  } while (0)

  // fragment addresses as LDS byte offsets: row base + swizzled chunk of k-step kk; tiles and stages are immediates
  const int sw = (l32 >> 1) & 7;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  uint32_t a_ad[4], b_ad[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    const int off = ((2 * kk + half) ^ sw) << 4;
    a_ad[kk] = lds0 + (wm * 128 + l32) * 128 + off;
    b_ad[kk] = lds0 + 65536 + (wn * 64 + l32) * 128 + off;
  }
#define MLPHS_DSREAD(dst, addr, imm) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
#define MLPHS_READ(fa, fb, s_, kk_)                               \
  do {                                                            \
    MLPHS_DSREAD(fa[0], a_ad[kk_], (s_) * 32768 + 0);             \
    MLPHS_DSREAD(fa[1], a_ad[kk_], (s_) * 32768 + 4096);          \
    MLPHS_DSREAD(fa[2], a_ad[kk_], (s_) * 32768 + 8192);          \
    MLPHS_DSREAD(fa[3], a_ad[kk_], (s_) * 32768 + 12288);         \
    MLPHS_DSREAD(fb[0], b_ad[kk_], (s_) * 32768 + 0);             \
    MLPHS_DSREAD(fb[1], b_ad[kk_], (s_) * 32768 + 4096);          \
  } while (0)
  // at most n_ LDS reads outstanding (they return in order); the fragments named become usable
#define MLPHS_WAIT(n_, fa, fb)                                                                           \
  asm volatile("s_waitcnt lgkmcnt(" #n_ ")"                                                              \
               : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1]))
#define MLPHS_MFMA(fa, fb)                                                                               \
  do {                                                                                                   \
    _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < TN; ++j_)                                                \
            acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i_]),    \
                                                                 __builtin_bit_cast(bf16x8, fb[j_]), acc[i_][j_], 0, 0, 0); \
  } while (0)
  // LD_: request the slice after next into the stage just released; NX_: read the next slice's first fragments
#define MLPHS_SLICE(s_, k2_, LD_, NX_)                                                                   \
  do {                                                                                                   \
    MLPHS_READ(qa, qb, s_, 1);                                                                           \
    MLPHS_WAIT(6, pa, pb);                                                                               \
    MLPHS_MFMA(pa, pb);                                                                                  \
    MLPHS_READ(pa, pb, s_, 2);                                                                           \
    MLPHS_WAIT(6, qa, qb);                                                                               \
    MLPHS_MFMA(qa, qb);                                                                                  \
    MLPHS_READ(qa, qb, s_, 3);                                                                           \
    MLPHS_WAIT(6, pa, pb);                                                                               \
    MLPHS_MFMA(pa, pb);                                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                                     \
    MLPHS_WAIT(0, qa, qb);                                                                               \
    asm volatile("s_barrier" ::: "memory");                                                              \
    if (LD_) MLPHS_FETCH(s_, (k2_) * 64);                                                                \
    if (NX_) MLPHS_READ(pa, pb, (s_) ^ 1, 0);                                                            \
    MLPHS_MFMA(qa, qb);                                                                                  \
  } while (0)

  const int nk = Kd / 64;                      // even and >= 2 (the launcher checks)
  MLPHS_FETCH(0, 0);
  MLPHS_FETCH(1, 64);
  asm volatile("s_waitcnt vmcnt(8)" ::: "memory");                 // slice 0 has landed, slice 1 may be in flight
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  u32x4 pa[4], pb[2], qa[4], qb[2];
  MLPHS_READ(pa, pb, 0, 0);
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {               // steady state without branches
    MLPHS_SLICE(0, kt + 2, 1, 1);
    MLPHS_SLICE(1, kt + 3, 1, 1);
  }
  MLPHS_SLICE(0, 0, 0, 1);                     // slice nk-2: nothing left to request
  MLPHS_SLICE(1, 0, 0, 0);                     // slice nk-1
#undef MLPHS_SLICE
#undef MLPHS_MFMA
#undef MLPHS_WAIT
#undef MLPHS_READ
#undef MLPHS_DSREAD
#undef MLPHS_FETCH

  float bcol[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bcol[j] = EPI == 1 ? 0.f : p.bias[tile_n * BN + wn * 64 + j * 32 + l32];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int lm = wm * 128 + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
      const int gm = tile_m * BM + lm;
      if (gm >= M) continue;
      const int src = sh_src[lm];
      const float* brow = EPI == 1 ? p.bias + static_cast<size_t>(sh_step[lm]) * p.N : p.bias;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int gn = tile_n * BN + wn * 64 + j * 32 + l32;
        const float c = acc[i][j][v] + (EPI == 1 ? brow[gn] : bcol[j]);
        if (EPI == 3) p.outf[static_cast<size_t>(src) * p.N + gn] = c;
        else p.outb[static_cast<size_t>(gm) * p.N + gn] = to_bf16_bits(silu(c));
      }
    }
  }
}

// true when kernel_hs can take the problem (otherwise the generic 256 x 256 kernel does)
inline bool hs_applicable(const Args& a) { return a.Kdim >= 128 && (a.Kdim / BK) % 2 == 0; }

template <int EPI, bool GATHER = false, int PM = 4, int PN = 8>
hipError_t prepare_hs() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel_hs<EPI, GATHER, PM, PN>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
}

template <int EPI, bool GATHER = false, int PM = 4, int PN = 8>
hipError_t launch_hs(const Args& a, int Rmax, hipStream_t st) {
  constexpr size_t shmem = 131072;
  const int tiles_m = (Rmax + 255) / 256, tiles_n = a.N / 256;
  const int patches = ((tiles_m + PM - 1) / PM) * ((tiles_n + PN - 1) / PN);
  const int grid = (patches * PM * PN + 7) / 8 * 8;
  hipLaunchKernelGGL((kernel_hs<EPI, GATHER, PM, PN>), dim3(grid), dim3(512), shmem, st, a);
  return hipGetLastError();
}

}  // namespace mlpgemm
