// Alternating-phase ("ping-pong") form of the 256 x 256 x 64 bf16 GEMM tile of mlp_gemm.h, built around
// v_mfma_f32_16x16x32_bf16.  Same operands, LDS layout, direct global->LDS loads and epilogue fusions as
// kernel_hs; what differs is how the eight wavefronts share the CU and when the loads are requested.
//
// A SIMD holds two wavefronts of the workgroup (wave and wave + 4).  The first four wavefronts form group 0,
// the other four group 1.  Every wavefront's work on a 64-wide slice is cut into four (memory, compute)
// phase pairs, one per 64 x 32 quadrant of its 128 x 64 share of the tile:
//     memory phase   ds_read_b128 of the fragments the next compute phase needs, and two direct loads
//     compute phase  16 MFMAs (256 matrix-pipe cycles) at raised wave priority, nothing else
// and a workgroup barrier closes every phase.  Group 1 runs one phase behind group 0 (it waits at one extra
// barrier before its first phase, group 0 at one extra barrier after its last), so on every SIMD one wavefront is
// in a compute phase while the other is in a memory phase: the matrix pipe always has exactly one wavefront
// feeding it and the LDS / load traffic of the other hides behind it, instead of all eight wavefronts reading
// fragments, issuing MFMAs and draining their loads at the same moments as they do in kernel_hs.
//
// Quadrant order (0,0) (0,1) (1,1) (1,0): consecutive quadrants share the A half or the B half, so a memory
// phase reads one new operand half only -- A0 (8 reads), B1 (4), A1 (8), and in the fourth phase the B0 of the
// NEXT slice (4), which sits in the other LDS stage.  The two B buffers swap roles from slice to slice.
//
// Loads.  A stage (64 KiB) is not released as a whole: each of its four regions -- the rows that are some
// wavefront's B0, A0, B1, A1 -- is free as soon as both groups have read it, and is refilled right then with the
// slice after next.  g = global phase index; group 0 runs the memory phase q of slice s at g = 8s + 2q, its
// compute phase at g + 1, group 1 one later:
//     region   last read (slice s)        refilled with slice s+2 in       first read of slice s+2
//     B0       memory phase 3 of s-1      memory phase 0 of s (g = 8s, +1)  8s+14
//     A0       memory phase 0             memory phase 1 (8s+2, +1)         8s+16
//     B1       memory phase 1             memory phase 2 (8s+4, +1)         8s+18
//     A1       memory phase 2             memory phase 3 (8s+6, +1)         8s+20
// so every load has 13 to 14 phases (more than a slice and a half) to land, the 64 loads of a slice are spread
// evenly over its eight phases (every wavefront issues two per memory phase: 16 loads of 8 rows cover the 128
// rows of a region), and no extra LDS is needed.  A wavefront's loads complete in order, and in steady state the
// region that is read next is always the one whose loads are 12 back in the wavefront's own sequence: every
// memory phase ends with s_waitcnt vmcnt(12), then lgkmcnt(0), then the barrier (the last two slices, which
// request nothing, count down 10, 8, 6, 4, 2, 0).
//
// Hazards: a region is refilled only after the barrier that follows its last read by either group (table above);
// a fragment register is overwritten by a later ds_read only after every MFMA that reads it has issued (program
// order; the LDS latency exceeds the operand read of an issued MFMA); there is no branch between a fragment
// read and its s_waitcnt (to the compiler an inline-asm read is complete when the statement ends, so a merge
// point in between could copy a register whose data is still on its way -- switches that remove reads or loads
// for timing experiments are therefore compile-time).  Every wavefront executes the same number of barriers.
#pragma once
#include "mlp_gemm.h"

namespace mlpgemm {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// DIAG (timing experiments only, results wrong): bit 0 = no fragment reads, bit 1 = no direct loads in the
// steady-state loop, bit 2 = no B fragment reads (a third of the LDS read traffic: what a layout that reads 128 KiB
// instead of 192 KiB per slice could gain at best); 3 leaves the MFMAs and barriers: what the schedule itself can
// reach on this chip
template <int EPI, bool GATHER = false, int DIAG = 0, int PM = 4, int PN = 8>
__global__ __launch_bounds__(512) void kernel_pp(Args p) {
  constexpr int BM = 256, BN = 256;
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
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // wavefront-uniform: the group branches below are scalar
  const int grp = wave >> 2;                     // 0: leads, 1: one phase behind
  const int wm = grp, wn = wave & 3;             // this wavefront's 128 x 64 share: rows wm*128.., columns wn*64..
  const int l16 = lane & 15, lq = lane >> 4;
  const int Kd = p.Kdim;
  const int nk = Kd / 64;                      // even and >= 2 (the launcher checks)
  // Direct loads: one wavefront instruction moves 8 rows x 128 B (lane -> row lane / 8, 16-byte chunk lane % 8 of
  // the LDS row; the chunk it fetches from global memory is that position XOR (LDS row >> 1) & 7).  Wavefront w
  // issues instructions u = 2w and 2w + 1 of each region's 16: B0 rows (u / 4) * 64 + (u % 4) * 8, B1 the same
  // + 32, A0 rows (u / 8) * 128 + (u % 8) * 8, A1 the same + 64.  The 8-row group's parity is that of u.
  const int lrow = lane >> 3;
  int ld_rowa[2], ld_rowb[2];                  // first LDS row of the two instructions (wavefront-uniform)
  const unsigned char *b0_src[2], *a0_src[2], *a1_src[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int u = 2 * wave + e;
    const int lchunk = (lane & 7) ^ ((4 * e + (lane >> 4)) & 7);
    ld_rowb[e] = (u >> 2) * 64 + (u & 3) * 8;
    ld_rowa[e] = (u >> 3) * 128 + (u & 7) * 8;
    b0_src[e] = reinterpret_cast<const unsigned char*>(p.Bt) +
                (static_cast<size_t>(tile_n) * BN + ld_rowb[e] + lrow) * Kd * 2 + 16 * lchunk;
    int r0 = tile_m * BM + ld_rowa[e] + lrow, r1 = r0 + 64;
    if (GATHER) {
      r0 = p.arow[r0 < M ? r0 : M - 1];
      r1 = p.arow[r1 < M ? r1 : M - 1];
    }
    a0_src[e] = reinterpret_cast<const unsigned char*>(p.A) + static_cast<size_t>(r0) * Kd * 2 + 16 * lchunk;
    a1_src[e] = reinterpret_cast<const unsigned char*>(p.A) + static_cast<size_t>(r1) * Kd * 2 + 16 * lchunk;
  }
  const size_t b1_off = static_cast<size_t>(32) * Kd * 2;

  __shared__ int sh_src[BM], sh_step[BM];        // epilogue bookkeeping, fetched ahead of the K loop (see kernel_hs)
  if (t < BM) {
    const int gm = tile_m * BM + t;
    const int src = p.rowidx[gm < M ? gm : M - 1];
    sh_src[t] = src;
    sh_step[t] = EPI == 1 ? p.krow[src] : 0;
  }

  // acc[i][ta][j][tb]: rows wm*128 + i*64 + ta*16 + (lane & 15), columns wn*64 + j*32 + tb*16 + 4*(lane >> 4) + v
  f32x4 acc[2][4][2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[i][a][j][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  typedef __attribute__((address_space(3))) void* lds_ptr;
  typedef const __attribute__((address_space(1))) void* gbl_ptr;
  // LDS map: A stage s at s * 32 KiB, B stage s at 64 KiB + s * 32 KiB; row r of a tile at r * 128 B, its 16-byte
  // chunk c at position c ^ ((r >> 1) & 7)
#define MLPPP_LD(src_, ldsoff_) \
  __builtin_amdgcn_global_load_lds((gbl_ptr)(src_), (lds_ptr)(smem + (ldsoff_)), 16, 0, 0)
  // the two loads of this wavefront into region B0 / A0 / B1 / A1 of stage s_, slice starting at element k0
#define MLPPP_LD_B0(s_, k0)                                                                              \
  do {                                                                                                   \
    MLPPP_LD(b0_src[0] + (k0) * 2, 65536 + (s_) * 32768 + ld_rowb[0] * 128);                             \
    MLPPP_LD(b0_src[1] + (k0) * 2, 65536 + (s_) * 32768 + ld_rowb[1] * 128);                             \
  } while (0)
#define MLPPP_LD_B1(s_, k0)                                                                              \
  do {                                                                                                   \
    MLPPP_LD(b0_src[0] + b1_off + (k0) * 2, 65536 + (s_) * 32768 + (ld_rowb[0] + 32) * 128);             \
    MLPPP_LD(b0_src[1] + b1_off + (k0) * 2, 65536 + (s_) * 32768 + (ld_rowb[1] + 32) * 128);             \
  } while (0)
#define MLPPP_LD_A0(s_, k0)                                                                              \
  do {                                                                                                   \
    MLPPP_LD(a0_src[0] + (k0) * 2, (s_) * 32768 + ld_rowa[0] * 128);                                     \
    MLPPP_LD(a0_src[1] + (k0) * 2, (s_) * 32768 + ld_rowa[1] * 128);                                     \
  } while (0)
#define MLPPP_LD_A1(s_, k0)                                                                              \
  do {                                                                                                   \
    MLPPP_LD(a1_src[0] + (k0) * 2, (s_) * 32768 + (ld_rowa[0] + 64) * 128);                              \
    MLPPP_LD(a1_src[1] + (k0) * 2, (s_) * 32768 + (ld_rowa[1] + 64) * 128);                              \
  } while (0)
#define MLPPP_LD_SLICE(s_, k0) \
  do { MLPPP_LD_B0(s_, k0); MLPPP_LD_A0(s_, k0); MLPPP_LD_B1(s_, k0); MLPPP_LD_A1(s_, k0); } while (0)

  // 16x16x32 fragment of rows r0..r0+15, k-step ks (32 wide): lane reads row r0 + (lane & 15), logical chunk 4*ks + (lane >> 4)
  const int sw = l16 >> 1;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
  uint32_t a_ad[2], b_ad[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int off = ((4 * ks + lq) ^ sw) << 4;
    a_ad[ks] = lds0 + (wm * 128 + l16) * 128 + off;
    b_ad[ks] = lds0 + 65536 + (wn * 64 + l16) * 128 + off;
  }
#define MLPPP_DSREAD(dst, addr, imm) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm))
  // fa[2*ta + ks]: A half i_ (64 rows) of stage s_
#define MLPPP_READ_A(s_, i_)                                                      \
  do {                                                                            \
    MLPPP_DSREAD(fa[0], a_ad[0], (s_) * 32768 + (i_) * 8192 + 0);                 \
    MLPPP_DSREAD(fa[1], a_ad[1], (s_) * 32768 + (i_) * 8192 + 0);                 \
    MLPPP_DSREAD(fa[2], a_ad[0], (s_) * 32768 + (i_) * 8192 + 2048);              \
    MLPPP_DSREAD(fa[3], a_ad[1], (s_) * 32768 + (i_) * 8192 + 2048);              \
    MLPPP_DSREAD(fa[4], a_ad[0], (s_) * 32768 + (i_) * 8192 + 4096);              \
    MLPPP_DSREAD(fa[5], a_ad[1], (s_) * 32768 + (i_) * 8192 + 4096);              \
    MLPPP_DSREAD(fa[6], a_ad[0], (s_) * 32768 + (i_) * 8192 + 6144);              \
    MLPPP_DSREAD(fa[7], a_ad[1], (s_) * 32768 + (i_) * 8192 + 6144);              \
  } while (0)
  // fb[2*tb + ks]: B half j_ (32 columns) of stage s_
#define MLPPP_READ_B(fb, s_, j_)                                                  \
  do {                                                                            \
    MLPPP_DSREAD(fb[0], b_ad[0], (s_) * 32768 + (j_) * 4096 + 0);                 \
    MLPPP_DSREAD(fb[1], b_ad[1], (s_) * 32768 + (j_) * 4096 + 0);                 \
    MLPPP_DSREAD(fb[2], b_ad[0], (s_) * 32768 + (j_) * 4096 + 2048);              \
    MLPPP_DSREAD(fb[3], b_ad[1], (s_) * 32768 + (j_) * 4096 + 2048);              \
  } while (0)
  // all LDS reads of this wavefront have returned; the fragments named become usable
#define MLPPP_WAIT_A()                                                                                   \
  asm volatile("s_waitcnt lgkmcnt(0)"                                                                    \
               : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fa[4]), "+v"(fa[5]), "+v"(fa[6]), "+v"(fa[7]))
#define MLPPP_WAIT_B(fb) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]))
  // the weights are the first MFMA operand: a lane then holds 4 consecutive output columns of one row
#define MLPPP_MFMA(i_, j_, fb)                                                                           \
  do {                                                                                                   \
    _Pragma("unroll") for (int ks_ = 0; ks_ < 2; ++ks_)                                                  \
        _Pragma("unroll") for (int ta_ = 0; ta_ < 4; ++ta_)                                              \
            _Pragma("unroll") for (int tb_ = 0; tb_ < 2; ++tb_)                                          \
                acc[i_][ta_][j_][tb_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                         \
                    __builtin_bit_cast(bf16x8, fb[2 * tb_ + ks_]), __builtin_bit_cast(bf16x8, fa[2 * ta_ + ks_]), \
                    acc[i_][ta_][j_][tb_], 0, 0, 0);                                                     \
  } while (0)
#define MLPPP_PHASE_END()                                                                                \
  do {                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    asm volatile("s_barrier" ::: "memory");                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  } while (0)
#define MLPPP_VMWAIT(n_) asm volatile("s_waitcnt vmcnt(" #n_ ")" ::: "memory")
#define MLPPP_COMPUTE(i_, j_, fb)                                                                        \
  do {                                                                                                   \
    __builtin_amdgcn_s_setprio(1);                                                                       \
    MLPPP_MFMA(i_, j_, fb);                                                                              \
    __builtin_amdgcn_s_setprio(0);                                                                       \
    MLPPP_PHASE_END();                                                                                   \
  } while (0)
  // One slice in stage s_: X holds its B0 on entry; on exit Y holds the next slice's B0 (NX_).  LD_: the four
  // regions of the stage are refilled with the slice that starts at element k2_ * 64 as they fall free.
  // W0_..W3_: loads that may still be outstanding at the end of each memory phase.
#define MLPPP_SLICE(s_, X, Y, k2_, LD_, NX_, W0_, W1_, W2_, W3_)                                         \
  do {                                                                                                   \
    if (!(DIAG & 1)) MLPPP_READ_A(s_, 0);                                                                \
    if (LD_ && !(DIAG & 2)) MLPPP_LD_B0(s_, (k2_) * 64);                                                 \
    MLPPP_WAIT_A();                                                                                      \
    MLPPP_VMWAIT(W0_);                                                                                   \
    MLPPP_PHASE_END();                                                                                   \
    MLPPP_COMPUTE(0, 0, X);                                                                              \
    if (!(DIAG & 5)) MLPPP_READ_B(Y, s_, 1);                                                             \
    if (LD_ && !(DIAG & 2)) MLPPP_LD_A0(s_, (k2_) * 64);                                                 \
    MLPPP_WAIT_B(Y);                                                                                     \
    MLPPP_VMWAIT(W1_);                                                                                   \
    MLPPP_PHASE_END();                                                                                   \
    MLPPP_COMPUTE(0, 1, Y);                                                                              \
    if (!(DIAG & 1)) MLPPP_READ_A(s_, 1);                                                                \
    if (LD_ && !(DIAG & 2)) MLPPP_LD_B1(s_, (k2_) * 64);                                                 \
    MLPPP_WAIT_A();                                                                                      \
    MLPPP_VMWAIT(W2_);                                                                                   \
    MLPPP_PHASE_END();                                                                                   \
    MLPPP_COMPUTE(1, 1, Y);                                                                              \
    if (NX_ && !(DIAG & 5)) MLPPP_READ_B(Y, (s_) ^ 1, 0);                                                \
    if (LD_ && !(DIAG & 2)) MLPPP_LD_A1(s_, (k2_) * 64);                                                 \
    MLPPP_WAIT_B(Y);                                                                                     \
    MLPPP_VMWAIT(W3_);                                                                                   \
    MLPPP_PHASE_END();                                                                                   \
    MLPPP_COMPUTE(1, 0, X);                                                                              \
  } while (0)

  MLPPP_LD_SLICE(0, 0);
  MLPPP_LD_SLICE(1, 64);
  MLPPP_VMWAIT(8);                                                 // slice 0 has landed, slice 1 may be in flight
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  u32x4 fa[8] = {}, bx[4] = {}, by[4] = {};
  int kt = 0;
  MLPPP_READ_B(bx, 0, 0);
  MLPPP_WAIT_B(bx);
  MLPPP_PHASE_END();                           // every wavefront holds its B0 of slice 0: that region may be refilled
  if (grp == 1) MLPPP_PHASE_END();             // group 1 starts one phase late
  for (; kt + 3 < nk; kt += 2) {
    MLPPP_SLICE(0, bx, by, kt + 2, 1, 1, 12, 12, 12, 12);
    MLPPP_SLICE(1, by, bx, kt + 3, 1, 1, 12, 12, 12, 12);
  }
  MLPPP_SLICE(0, bx, by, 0, 0, 1, 10, 8, 6, 4);     // slice nk-2: nothing left to request
  MLPPP_SLICE(1, by, bx, 0, 0, 0, 2, 0, 0, 0);      // slice nk-1
  if (grp == 0) MLPPP_PHASE_END();             // group 0 waits for group 1's last phase: equal barrier counts
#undef MLPPP_SLICE
#undef MLPPP_COMPUTE
#undef MLPPP_VMWAIT
#undef MLPPP_LD_SLICE
#undef MLPPP_LD_A1
#undef MLPPP_LD_A0
#undef MLPPP_LD_B1
#undef MLPPP_LD_B0
#undef MLPPP_LD
#undef MLPPP_PHASE_END
#undef MLPPP_MFMA
#undef MLPPP_WAIT_B
#undef MLPPP_WAIT_A
#undef MLPPP_READ_B
#undef MLPPP_READ_A
#undef MLPPP_DSREAD

  // ---- epilogue: a lane holds, per 16 x 16 tile, 4 consecutive columns of one row
  f32x4 bcol[2][2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int b = 0; b < 2; ++b)
      bcol[j][b] = EPI == 1 ? f32x4{0.f, 0.f, 0.f, 0.f}
                            : *reinterpret_cast<const f32x4*>(p.bias + tile_n * BN + wn * 64 + j * 32 + b * 16 + 4 * lq);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int lm = wm * 128 + i * 64 + a * 16 + l16;
      const int gm = tile_m * BM + lm;
      if (gm >= M) continue;
      const int src = sh_src[lm];
      const float* brow = EPI == 1 ? p.bias + static_cast<size_t>(sh_step[lm]) * p.N : p.bias;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int gn = tile_n * BN + wn * 64 + j * 32 + b * 16 + 4 * lq;
          f32x4 c = acc[i][a][j][b];
          if (EPI == 1) c += *reinterpret_cast<const f32x4*>(brow + gn);
          else c += bcol[j][b];
          if (EPI == 3) {
            *reinterpret_cast<f32x4*>(p.outf + static_cast<size_t>(src) * p.N + gn) = c;
          } else {
            uint2 o;
            o.x = to_bf16_bits(silu(c[0])) | (static_cast<uint32_t>(to_bf16_bits(silu(c[1]))) << 16);
            o.y = to_bf16_bits(silu(c[2])) | (static_cast<uint32_t>(to_bf16_bits(silu(c[3]))) << 16);
            *reinterpret_cast<uint2*>(p.outb + static_cast<size_t>(gm) * p.N + gn) = o;
          }
        }
      }
    }
  }
}

template <int EPI, bool GATHER = false, int DIAG = 0, int PM = 4, int PN = 8>
hipError_t prepare_pp() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&kernel_pp<EPI, GATHER, DIAG, PM, PN>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 131072);
}

// Takes what kernel_hs takes (hs_applicable); prepare_pp<...>() must have run once for the instantiation.
template <int EPI, bool GATHER = false, int DIAG = 0, int PM = 4, int PN = 8>
hipError_t launch_pp(const Args& a, int Rmax, hipStream_t st) {
  const int tiles_m = (Rmax + 255) / 256, tiles_n = a.N / 256;
  const int patches = ((tiles_m + PM - 1) / PM) * ((tiles_n + PN - 1) / PN);
  const int grid = (patches * PM * PN + 7) / 8 * 8;
  hipLaunchKernelGGL((kernel_pp<EPI, GATHER, DIAG, PM, PN>), dim3(grid), dim3(512), 131072, st, a);
  return hipGetLastError();
}

}  // namespace mlpgemm
