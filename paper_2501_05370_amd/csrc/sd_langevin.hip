// One speculative window of unadjusted Langevin on a Gaussian-mixture energy, fused in one launch.
//
// Paper: Sec. 5 and Alg. "Speculative Sampling for Unadjusted Langevin Diffusion", frozen-gradient
// proxy (grad E^(x_{n+j}) = grad E(x_n)):
//   draft    y~_{j} = y~_{j-1} - gamma g0 + sqrt(2 gamma) z_j,          g0 = grad E(x_n)
//   target   mean     y~_{j-1} - gamma grad E(y~_{j-1})
//   Delta_j = sqrt(gamma/2) (grad E(y~_{j-1}) - g0),  accept iff log u <= min(0, -z.Delta - |Delta|^2/2)
//   reject:  x_out = y~_{j-1} - gamma grad E(y~_{j-1}) + sqrt(2 gamma) (z - 2 (z.Delta/|Delta|^2) Delta)
// with E(x) = -log sum_m w_m N(x; mu_m, s^2 I), grad E = (x - sum_m r_m(x) mu_m) / s^2.
//
// Three kernels.  For d <= 1024 a WAVEFRONT owns a chain (langevin_window_wave_kernel, further down); for
// larger d a workgroup does (langevin_window_kernel, next): a thread owns CPT groups of four consecutive
// coordinates (= one Philox block each), keeps the window state, the frozen gradient and its slice of
// the mixture means in registers, and walks the window positions in order; because the whole chain
// lives in one workgroup the walk simply stops at the first rejection, so no work is spent on drafts
// that would be discarded.  Per position: 16 logit partial sums and the two dot products are reduced
// over the workgroup in fp64.  The phi^4 lattice energy has kernels of its own at the end of the file.
#include <hip/hip_runtime.h>

#include <cmath>

#include "sd_internal.h"
#include "sd_lanes.h"
#include "sd_rng.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

struct LangevinArgs {
  const float* x;
  const int32_t* n;
  const int64_t* id;
  const float* means;   // [M,d]
  const float* logw;    // [M]
  float* x_out;
  int32_t* adv;
  uint8_t* rej;
  float *logratio, *logu;
  const int32_t* active;
  int32_t* queue;       // chain dispenser of the wavefront kernel: the next chain to hand out (zeroed ahead of the launch)
  int max_windows;      // 1: one window per chain (sd_langevin_window); > 1: windows back to back (sd_langevin_run)
  int32_t* n_out;       // run mode: the step each chain reached
  unsigned long long* counters;   // run mode, optional: sum adv, chain-windows, rejections, launches, sum Kt
  int B, d, K, T, M;
  uint64_t seed;
  double gamma, inv_s2, inv_tau;
};

__device__ __forceinline__ double wave_sum(double v) { return sdlane::wave_sum(v); }

// v of lane (lane ^ mask), mask a single bit known at compile time after unrolling
__device__ __forceinline__ double dpp_xor(double v, int mask) {
  switch (mask) {
    case 1: return sdlane::lane_xor<1>(v);
    case 2: return sdlane::lane_xor<2>(v);
    case 4: return sdlane::lane_xor<4>(v);
    case 8: return sdlane::lane_xor<8>(v);
    case 16: return sdlane::lane_xor<16>(v);
    default: return sdlane::lane_xor<32>(v);
  }
}

// CPT: float4 groups per thread; MMAX: compile-time bound on the number of components.
template <int CPT, int MMAX>
__global__ __launch_bounds__(kThreads) void langevin_window_kernel(LangevinArgs p) {
  __shared__ double sh_part[kWaves][MMAX + 2];
  __shared__ double sh_r[MMAX];

  const int b = blockIdx.x;
  const int Bact = p.active ? min(p.B, max(0, *p.active)) : p.B;
  if (b >= Bact) return;                       // uniform over the workgroup
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int n = p.n[b];
  const int Kt = max(0, min(p.K, p.T - n));
  const int64_t id = p.id[b];
  const int d = p.d, M = p.M;
  const double gamma = p.gamma, inv_s2 = p.inv_s2;
  const double sq2g = sqrt(2.0 * gamma), sqg2 = sqrt(0.5 * gamma);

  // ---- my coordinates, my slice of the means
  bool own[CPT][4];
  double cur[CPT][4];          // y~_{j-1}: the state the target gradient is evaluated at
  float mu[CPT][MMAX][4];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int i0 = 4 * (t + kThreads * c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      own[c][e] = i0 + e < d;
      cur[c][e] = own[c][e] ? static_cast<double>(p.x[static_cast<int64_t>(b) * d + i0 + e]) : 0.0;
#pragma unroll
      for (int m = 0; m < MMAX; ++m)
        mu[c][m][e] = (own[c][e] && m < M) ? p.means[static_cast<int64_t>(m) * d + i0 + e] : 0.f;
    }
  }

  // grad E at `cur` for my coordinates.  Uniform control flow: called by every thread.
  auto gradient = [&](double g[CPT][4]) {
    double q[MMAX];
#pragma unroll
    for (int m = 0; m < MMAX; ++m) {
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const double df = cur[c][e] - static_cast<double>(mu[c][m][e]);
          acc = fma(df, df, acc);              // unowned coordinates contribute 0 - 0
        }
      q[m] = wave_sum(acc);
    }
    __syncthreads();                           // previous readers of sh_part / sh_r are done
    if (lane == 0) {
#pragma unroll
      for (int m = 0; m < MMAX; ++m) sh_part[wave][m] = q[m];
    }
    __syncthreads();
    if (t < 64) {                              // first wavefront: softmax over the components
      double logit = -INFINITY;
      if (t < M) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) tot += sh_part[w][t];
        logit = static_cast<double>(p.logw[t]) - 0.5 * tot * inv_s2;
      }
      double mx = logit;
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) mx = fmax(mx, dpp_xor(mx, s));
      const double ex = t < M ? exp(logit - mx) : 0.0;
      const double sum = wave_sum(ex);
      if (t < M) sh_r[t] = ex / sum;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double bar = 0.0;
#pragma unroll
        for (int m = 0; m < MMAX; ++m)
          if (m < M) bar = fma(sh_r[m], static_cast<double>(mu[c][m][e]), bar);
        g[c][e] = (cur[c][e] - bar) * inv_s2;
      }
  };

  double g0[CPT][4];
  gradient(g0);

  int jr = -1;
  double coef = 0.0;
  double gj[CPT][4];
  float z[CPT][4];
  double dl[CPT][4];
  for (int j = 0; j < Kt; ++j) {               // tests state n+j+1; Kt is uniform over the workgroup
    const uint32_t k1 = static_cast<uint32_t>(n + j + 1);
#pragma unroll
    for (int c = 0; c < CPT; ++c)
      sdrng::normal4(p.seed, id, k1, sdrng::kStreamNoise, static_cast<uint32_t>(t + kThreads * c), z[c]);
    double lr = 0.0, lu = 0.0;
    bool reject = false;
    if (j > 0) {                               // position 1: the target gradient IS g0, Delta = 0
      gradient(gj);
      double a1 = 0.0, a2 = 0.0;
#pragma unroll
      for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dl[c][e] = own[c][e] ? sqg2 * (gj[c][e] - g0[c][e]) : 0.0;
          a1 = fma(static_cast<double>(z[c][e]), dl[c][e], a1);
          a2 = fma(dl[c][e], dl[c][e], a2);
        }
      a1 = wave_sum(a1);
      a2 = wave_sum(a2);
      __syncthreads();
      if (lane == 0) { sh_part[wave][MMAX] = a1; sh_part[wave][MMAX + 1] = a2; }
      __syncthreads();
      double S1 = 0.0, S2 = 0.0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) { S1 += sh_part[w][MMAX]; S2 += sh_part[w][MMAX + 1]; }
      lr = (-S1 - 0.5 * S2) * p.inv_tau;
      lu = sdrng::log_uniform(p.seed, id, k1);
      reject = !(S2 == 0.0 || (lr == lr && lu <= fmin(0.0, lr)));   // a log-ratio that is not a number rejects
      coef = S2 > 0.0 ? S1 / S2 : 0.0;
    } else {
      lu = sdrng::log_uniform(p.seed, id, k1);
    }
    if (t == 0) {
      if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lr);
      if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lu);
    }
    if (reject) {                              // every thread holds the same totals: uniform branch
      jr = j;
#pragma unroll
      for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (own[c][e])
            cur[c][e] = cur[c][e] - gamma * gj[c][e] +
                        sq2g * (static_cast<double>(z[c][e]) - 2.0 * coef * dl[c][e]);
      break;
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (own[c][e])                         // unowned slots stay 0 so they never reach a sum
          cur[c][e] = cur[c][e] - gamma * g0[c][e] + sq2g * static_cast<double>(z[c][e]);
  }

  if (t == 0) {
    p.adv[b] = jr >= 0 ? jr + 1 : Kt;
    if (p.rej) p.rej[b] = jr >= 0 ? 1 : 0;
    const int jdone = jr >= 0 ? jr + 1 : Kt;   // positions not reached report 0
    for (int j = jdone; j < p.K; ++j) {
      if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = 0.f;
      if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = 0.f;
    }
  }
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int i0 = 4 * (t + kThreads * c);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (own[c][e]) p.x_out[static_cast<int64_t>(b) * d + i0 + e] = static_cast<float>(cur[c][e]);
  }
}

// ---------------------------------------------------------------------------------------------
// One WAVEFRONT per chain (d <= 1024 * CPT/4): no workgroup barrier on the walk at all.
// A lane owns CPT groups of four coordinates; the mixture means sit in LDS as fp64, once per workgroup
// (its kWaveChains wavefronts share them; the workgroups stay resident for the whole launch and their
// wavefronts draw chains from a counter).  Logits use  log w_m + (x.mu_m - |mu_m|^2/2)/s^2  (the |x|^2
// term cancels in the softmax), so a position costs two passes over the means: 16 dot products and the
// responsibility-weighted mean.  The 16 per-lane partial dot products are reduced with a transposed
// butterfly (values are exchanged in halves, 17 exchanges instead of 96, all of them DPP moves or row
// swaps in the vector ALU); responsibilities are then broadcast through scalar registers.
// RUN: the chain's windows follow each other inside the kernel (sd_langevin_run).
// ---------------------------------------------------------------------------------------------
constexpr int kWaveChains = 8;             // chains (wavefronts) per workgroup: one workgroup fills a CU at 2 per SIMD
constexpr int kWaveM = 16;                 // components handled by the transposed reduction


// in: 16 per-lane partial sums; out: total of value ((lane >> 2) & 15), on every lane
__device__ __forceinline__ double reduce16_transposed(double (&a)[16], int lane) {
  (void)lane;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = sdlane::halving_add<32>(a[i], a[i + 8]);
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = sdlane::halving_add<16>(a[i], a[i + 4]);
#pragma unroll
  for (int i = 0; i < 2; ++i) a[i] = sdlane::halving_add<8>(a[i], a[i + 2]);
  a[0] = sdlane::halving_add<4>(a[0], a[1]);
  a[0] += sdlane::lane_xor<2>(a[0]);
  a[0] += sdlane::lane_xor<1>(a[0]);
  return a[0];
}

__device__ __forceinline__ double readlane_f64(double v, int src_lane) {
  const long long bits = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane(static_cast<int>(bits), src_lane);
  const int hi = __builtin_amdgcn_readlane(static_cast<int>(bits >> 32), src_lane);
  return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}

// WHOLE: d is a multiple of 4, so a group of four coordinates is inside d or outside it as a whole (one mask
// per group instead of four).
template <int CPT, bool WHOLE, bool RUN>
__global__ __launch_bounds__(64 * kWaveChains, 2) void langevin_window_wave_kernel(LangevinArgs p, int dpad) {
  // [kWaveM][dpad] as fp64 (rows beyond M and the pad are 0): converted once here instead of once per use --
  // the logit pass is one FMA per table element, and a conversion beside each would be a fifth of all
  // vector instructions of the kernel.  16 x 1024 doubles = 128 KiB: one workgroup of 8 wavefronts per CU.
  extern __shared__ __align__(16) double sh_mu[];
  __shared__ double sh_hn[kWaveM];                         // |mu_m|^2 / 2
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int d = p.d, M = p.M;
  // Rows are read as whole float4s through this view, indexed in units of 16 bytes: with the row stride a
  // run-time number of floats the compiler cannot see that a row starts 16-byte aligned and splits every
  // 128-bit LDS read into 32-bit pairs, which are slower and collide on the banks.
  // Row layout: a row has kRow = 256 * CPT doubles; the four coordinates 4 g .. 4 g + 3 of group g = lane + 64 c
  // sit as two halves, (e = 0, 1) at c * 256 + 2 * lane and (e = 2, 3) at c * 256 + 128 + 2 * lane, so that each
  // of the two 128-bit reads of a group is contiguous over the lanes (conflict-free, and the row stride is a
  // compile-time multiple of 16 bytes).
  constexpr int kRow = 256 * CPT;
  const double2* sh_mu2 = reinterpret_cast<const double2*>(sh_mu);

  for (int idx = t; idx < kWaveM * kRow; idx += 64 * kWaveChains) {
    const int m = idx / kRow, i = idx % kRow;            // i: coordinate
    const int c = i >> 8, ln = (i & 255) >> 2, e = i & 3;
    const int pos = c * 256 + (e < 2 ? 2 * ln + e : 128 + 2 * ln + (e - 2));
    sh_mu[m * kRow + pos] = (m < M && i < d) ? static_cast<double>(p.means[static_cast<int64_t>(m) * d + i]) : 0.0;
  }
  __syncthreads();
  if (wave == 0) {                                         // half squared norms, fp64
    double part[16];
#pragma unroll
    for (int m = 0; m < kWaveM; ++m) {
      double acc = 0.0;
      for (int i = lane; i < kRow; i += 64) {
        const double v = sh_mu[m * kRow + i];
        acc = fma(v, v, acc);
      }
      part[m] = acc;
    }
    const double tot = reduce16_transposed(part, lane);
    if ((lane & 3) == 0) sh_hn[lane >> 2] = 0.5 * tot;
  }
  __syncthreads();                                         // last workgroup-wide barrier

  const int Bact = p.active ? min(p.B, max(0, *p.active)) : p.B;
  const double gamma = p.gamma, inv_s2 = p.inv_s2;
  const double sq2g = sqrt(2.0 * gamma), sqg2 = sqrt(0.5 * gamma), inv_sqg2 = 1.0 / sqg2;
  const int my_m = lane >> 2;                              // component this lane holds after a reduction
  const double my_logw = my_m < M ? static_cast<double>(p.logw[my_m]) : 0.0;
  const double my_hn = sh_hn[my_m];

  // The workgroup keeps its copy of the means for the whole launch (the table is staged once per resident
  // workgroup, not once per four chains) and its wavefronts, independent from here on, take chains one at a
  // time from a counter: a chain's window ends at its first rejection, so the work per chain varies by an
  // order of magnitude and a fixed split would leave most of the chip waiting for the unluckiest wavefront.
  constexpr bool run = RUN;                                // windows back to back: the chain stays in registers
  unsigned long long acc_adv = 0, acc_win = 0, acc_rej = 0, acc_kt = 0;   // run mode: this wavefront's share of the counters
  for (;;) {
  int ticket = 0;
  if (lane == 0) ticket = atomicAdd(&p.queue[0], 1);
  const int b = __builtin_amdgcn_readfirstlane(ticket);
  if (b >= Bact) break;
  int n = p.n[b];
  const int64_t id = p.id[b];

  bool own[CPT][4];
  double cur[CPT][4];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int i0 = 4 * (lane + 64 * c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      own[c][e] = WHOLE ? i0 < d : i0 + e < d;
      cur[c][e] = own[c][e] ? static_cast<double>(p.x[static_cast<int64_t>(b) * d + i0 + e]) : 0.0;
    }
  }

  // grad E at `cur` for my coordinates
  auto gradient = [&](double g[CPT][4]) {
    double dot[16];
#pragma unroll
    for (int m = 0; m < kWaveM; ++m) dot[m] = 0.0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {                        // 16 independent accumulation chains
      const int g4 = lane + 64 * c;
      if (4 * g4 < dpad) {
#pragma unroll
        for (int m = 0; m < kWaveM; ++m) {
          const double2 lo = sh_mu2[m * (kRow / 2) + c * 128 + lane], hi = sh_mu2[m * (kRow / 2) + c * 128 + 64 + lane];
          dot[m] = fma(cur[c][0], lo.x, dot[m]);
          dot[m] = fma(cur[c][1], lo.y, dot[m]);
          dot[m] = fma(cur[c][2], hi.x, dot[m]);
          dot[m] = fma(cur[c][3], hi.y, dot[m]);
        }
      }
    }
    const double tot = reduce16_transposed(dot, lane);     // x . mu_{my_m}
    double logit = my_m < M ? my_logw + (tot - my_hn) * inv_s2 : -INFINITY;
    double mx = logit;
#pragma unroll
    for (int s = 4; s <= 32; s <<= 1) mx = fmax(mx, dpp_xor(mx, s));
    const double ex = my_m < M ? exp(logit - mx) : 0.0;
    double sum = ex;
#pragma unroll
    for (int s = 4; s <= 32; s <<= 1) sum += dpp_xor(sum, s);
    const double r_mine = ex / sum;
    double bar[CPT][4];
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) bar[c][e] = 0.0;
#pragma unroll
    for (int m = 0; m < kWaveM; ++m) {
      const double r = readlane_f64(r_mine, 4 * m);        // uniform: lives in scalar registers
      // a component whose responsibility is below 1e-25 moves no coordinate of the weighted mean by more
      // than 1e-25 |mu|, far below the last bit of anything downstream: its pass over the means is skipped
      // (uniform branch).  Well-separated mixtures leave one or two components per state.
      if (r < 1e-25) continue;
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int g4 = lane + 64 * c;
        if (4 * g4 < dpad) {
          const double2 lo = sh_mu2[m * (kRow / 2) + c * 128 + lane], hi = sh_mu2[m * (kRow / 2) + c * 128 + 64 + lane];
          bar[c][0] = fma(r, lo.x, bar[c][0]);
          bar[c][1] = fma(r, lo.y, bar[c][1]);
          bar[c][2] = fma(r, hi.x, bar[c][2]);
          bar[c][3] = fma(r, hi.y, bar[c][3]);
        }
      }
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) g[c][e] = (cur[c][e] - bar[c][e]) * inv_s2;
  };

  int Kt = 0, jr = -1;
  for (int w = 0; w < (RUN ? p.max_windows : 1); ++w) {    // every window advances the chain by at least one step
  Kt = max(0, min(p.K, p.T - n));
  if ((RUN || w > 0) && Kt == 0) break;                    // the chain has reached T (a chain handed over at T: no window)
  double g0[CPT][4];
  gradient(g0);

  // log u of the window's positions: lane j draws position j + 1 (the window has at most 64), once per
  // window; a draw per position would cost every lane a Philox block and an fp64 log each time
  const double lu_mine = lane < Kt ? sdrng::log_uniform(p.seed, id, static_cast<uint32_t>(n + lane + 1)) : 0.0;

  jr = -1;
  double coef = 0.0;
  double dl[CPT][4];                                       // gradient at the draft, then Delta
  float z[CPT][4];
  for (int j = 0; j < Kt; ++j) {                           // Kt is uniform over the wavefront
    const uint32_t k1 = static_cast<uint32_t>(n + j + 1);
    double lr = 0.0;
    bool reject = false;
    if (j > 0) gradient(dl);                               // position 1: the target gradient IS g0
    // the noise and the uniform are drawn after the gradient, which is the register-hungry part
    // Coordinates past d (the tail of the last group) get no noise: their state starts at 0 and the means table
    // is 0 there, so state, gradients and Delta stay exactly 0 and need no masking anywhere else.
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      sdrng::normal4(p.seed, id, k1, sdrng::kStreamNoise, static_cast<uint32_t>(lane + 64 * c), z[c]);
#pragma unroll
      for (int e = 0; e < 4; ++e) z[c][e] = own[c][e] ? z[c][e] : 0.f;
    }
    const double lu = readlane_f64(lu_mine, j);
    if (j > 0) {
      double a1 = 0.0, a2 = 0.0;
#pragma unroll
      for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dl[c][e] = sqg2 * (dl[c][e] - g0[c][e]);
          a1 = fma(static_cast<double>(z[c][e]), dl[c][e], a1);
          a2 = fma(dl[c][e], dl[c][e], a2);
        }
      const double S1 = wave_sum(a1), S2 = wave_sum(a2);
      lr = (-S1 - 0.5 * S2) * p.inv_tau;
      reject = !(S2 == 0.0 || (lr == lr && lu <= fmin(0.0, lr)));   // a log-ratio that is not a number rejects
      coef = S2 > 0.0 ? S1 / S2 : 0.0;
    }
    if (lane == 0) {
      if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lr);
      if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lu);
    }
    if (reject) {                                          // all lanes hold the same totals
      jr = j;
#pragma unroll
      for (int c = 0; c < CPT; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          cur[c][e] = cur[c][e] - gamma * (g0[c][e] + dl[c][e] * inv_sqg2) +   // target gradient = g0 + Delta / sqrt(gamma/2)
                      sq2g * (static_cast<double>(z[c][e]) - 2.0 * coef * dl[c][e]);
      break;
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        cur[c][e] = cur[c][e] - gamma * g0[c][e] + sq2g * static_cast<double>(z[c][e]);
  }

  if (run) {
    // what sd_advance and the next sd_langevin_window would do: the step count moves on and the state passes
    // through fp32, so a run is bit for bit the window entry point applied again and again
    const int jdone = jr >= 0 ? jr + 1 : Kt;
    n += jdone;
    acc_adv += jdone; acc_win += 1; acc_rej += jr >= 0 ? 1 : 0; acc_kt += Kt;
#pragma unroll
    for (int c = 0; c < CPT; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) cur[c][e] = static_cast<double>(static_cast<float>(cur[c][e]));
  }
  }                                                        // next window of this chain

  if (lane == 0) {
    if (run) {
      p.n_out[b] = n;
    } else {
      p.adv[b] = jr >= 0 ? jr + 1 : Kt;
      if (p.rej) p.rej[b] = jr >= 0 ? 1 : 0;
      const int jdone = jr >= 0 ? jr + 1 : Kt;
      for (int j = jdone; j < p.K; ++j) {
        if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = 0.f;
        if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = 0.f;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int i0 = 4 * (lane + 64 * c);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (own[c][e]) p.x_out[static_cast<int64_t>(b) * d + i0 + e] = static_cast<float>(cur[c][e]);
  }
  }                                                        // next chain of this wavefront
  if (run && p.counters && lane == 0 && acc_win) {
    atomicAdd(&p.counters[0], acc_adv);
    atomicAdd(&p.counters[1], acc_win);
    atomicAdd(&p.counters[2], acc_rej);
    atomicAdd(&p.counters[4], acc_kt);
  }
}

// The chain dispenser starts every launch at zero: a one-thread kernel ahead of the launch (a kernel, not a
// memset, so that the sequence can be captured in a HIP graph), never a rewind at the end of the previous one --
// a launch that does not run to its end must not leave the next call without chains.
__global__ void reset_dispenser_kernel(int32_t* queue) { queue[0] = 0; }

// run mode: one launch counts as one entry of the `windows` counter
__global__ void bump_launches_kernel(unsigned long long* counters) { counters[3] += 1; }

template <int CPT, bool WHOLE, bool RUN>
hipError_t prepare_wave() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&langevin_window_wave_kernel<CPT, WHOLE, RUN>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
}

// prepare_wave<...>() has run for every instantiation when the context was created (sdi::langevin_prepare);
// `resident` = workgroups the chip holds at once (one per CU), from the same call.
template <int CPT, bool WHOLE, bool RUN>
hipError_t launch_wave(const LangevinArgs& p, int dpad, int resident, hipStream_t st) {
  const size_t shmem = sizeof(double) * kWaveM * static_cast<size_t>(256 * CPT);
  const int groups = (p.B + kWaveChains - 1) / kWaveChains;
  const unsigned grid = static_cast<unsigned>(groups < resident ? groups : resident);
  hipLaunchKernelGGL(reset_dispenser_kernel, dim3(1), dim3(1), 0, st, p.queue);
  hipLaunchKernelGGL((langevin_window_wave_kernel<CPT, WHOLE, RUN>), dim3(grid), dim3(64 * kWaveChains), shmem, st, p, dpad);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// phi^4 lattice energy on an L x L periodic grid (Langevin appendix, table of sampling metrics):
//   E(x) = (beta/2) sum over ordered neighbour pairs (x_i - x_j)^2 + sum_i (x_i^2 - 1)^2,
//   grad E_i = 2 beta (4 x_i - four neighbours) + 4 x_i (x_i^2 - 1).
// G lanes work on one chain (G = power of two >= d/4, one Philox block of four sites per lane),
// 64/G chains share a wavefront and 256/G a workgroup.  The chain's state is mirrored in a
// wavefront-private slice of LDS for the neighbour reads; no workgroup barrier is used, since the
// chains of a workgroup leave their walks at different positions.  A wavefront walks until none
// of its chains is alive; a chain that has rejected or finished is masked.
// ---------------------------------------------------------------------------------------------
struct Phi4Args {
  const float* x;
  const int32_t* n;
  const int64_t* id;
  float* x_out;
  int32_t* adv;
  uint8_t* rej;
  float *logratio, *logu;
  const int32_t* active;
  int B, d, L, K, T;
  uint64_t seed;
  double gamma, beta, inv_tau;
  int max_windows;                 // sd_langevin_run_phi4: windows per chain at most
  int32_t* n_out;                  //   the step each chain reached
  unsigned long long* counters;    //   optional: sum adv, chain-windows, rejections, launches, sum Kt
};

template <int G>
__device__ __forceinline__ double group_sum_f64(double v) {
#pragma unroll
  for (int s = G / 2; s >= 1; s >>= 1) v += dpp_xor(v, s);
  return v;
}

template <int G>
__global__ __launch_bounds__(256) void phi4_window_kernel(Phi4Args p) {
  constexpr int CPWV = 64 / G;                       // chains per wavefront
  extern __shared__ __align__(16) double sh_x[];     // [256 / G][d]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int sub = lane / G, gl = lane % G;
  const int slot = wave * CPWV + sub;
  const int Bact = p.active ? min(p.B, max(0, *p.active)) : p.B;
  const int b_raw = blockIdx.x * (4 * CPWV) + slot;
  const bool valid = b_raw < Bact;
  const int b = valid ? b_raw : 0;
  const int d = p.d, L = p.L;
  const int n = valid ? p.n[b] : 0;
  const int Kt = valid ? max(0, min(p.K, p.T - n)) : 0;
  const int64_t id = valid ? p.id[b] : 0;
  const double gamma = p.gamma, beta2 = 2.0 * p.beta;
  const double sq2g = sqrt(2.0 * gamma), sqg2 = sqrt(0.5 * gamma), inv_sqg2 = 1.0 / sqg2;
  double* xs = sh_x + static_cast<size_t>(slot) * d;

  bool own[4];
  int nb[4][4];
  double cur[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int s = 4 * gl + e;
    own[e] = s < d;
    const int sc = own[e] ? s : 0;
    const int r = sc / L, c = sc % L;
    nb[e][0] = ((r + L - 1) % L) * L + c;
    nb[e][1] = ((r + 1) % L) * L + c;
    nb[e][2] = r * L + (c + L - 1) % L;
    nb[e][3] = r * L + (c + 1) % L;
    cur[e] = (valid && own[e]) ? static_cast<double>(p.x[static_cast<int64_t>(b) * d + s]) : 0.0;
  }

  // grad E at `cur`: mirror the state in LDS, then read the four neighbours.  Writers and readers
  // are lanes of one wavefront and the two accesses are separate instructions in program order.
  auto gradient = [&](double g[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (own[e]) xs[4 * gl + e] = cur[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      double v = 0.0;
      if (own[e]) {
        const double s4 = xs[nb[e][0]] + xs[nb[e][1]] + xs[nb[e][2]] + xs[nb[e][3]];
        v = beta2 * (4.0 * cur[e] - s4) + 4.0 * cur[e] * (cur[e] * cur[e] - 1.0);
      }
      g[e] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                 // reads done before the next mirror overwrites
  };

  double g0[4];
  gradient(g0);

  int jr = -1;
  double lu_batch = 0.0;                             // log u of position (j - j % G) + gl + 1, drawn G positions at a time
  for (int j = 0; j < p.K; ++j) {
    const bool alive = valid && j < Kt && jr < 0;
    if (__ballot(alive) == 0ull) break;              // uniform over the wavefront
    const uint32_t k1 = static_cast<uint32_t>(n + j + 1);
    float z[4];
    sdrng::normal4(p.seed, id, k1, sdrng::kStreamNoise, static_cast<uint32_t>(gl), z);
    if (j % G == 0) lu_batch = sdrng::log_uniform(p.seed, id, static_cast<uint32_t>(n + j + gl + 1));   // j is uniform
    const double lu = __shfl(lu_batch, sub * G + j % G, 64);
    double lr = 0.0, coef = 0.0;
    bool reject = false;
    double dl[4] = {0.0, 0.0, 0.0, 0.0};
    if (j > 0) {                                     // position 1: the target gradient IS g0
      gradient(dl);                                  // every lane of the wavefront takes part
      double a1 = 0.0, a2 = 0.0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dl[e] = (own[e] && alive) ? sqg2 * (dl[e] - g0[e]) : 0.0;
        a1 = fma(static_cast<double>(z[e]), dl[e], a1);
        a2 = fma(dl[e], dl[e], a2);
      }
      const double S1 = group_sum_f64<G>(a1), S2 = group_sum_f64<G>(a2);
      lr = (-S1 - 0.5 * S2) * p.inv_tau;
      reject = alive && !(S2 == 0.0 || (lr == lr && lu <= fmin(0.0, lr)));
      coef = S2 > 0.0 ? S1 / S2 : 0.0;
    }
    if (alive && gl == 0) {
      if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lr);
      if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = static_cast<float>(lu);
    }
    if (alive) {
      if (reject) {
        jr = j;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (own[e])                                // target gradient = g0 + Delta / sqrt(gamma/2)
            cur[e] = cur[e] - gamma * (g0[e] + dl[e] * inv_sqg2) + sq2g * (static_cast<double>(z[e]) - 2.0 * coef * dl[e]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (own[e]) cur[e] = cur[e] - gamma * g0[e] + sq2g * static_cast<double>(z[e]);
      }
    }
  }

  if (!valid) return;
  const int jdone = jr >= 0 ? jr + 1 : Kt;
  if (gl == 0) {
    p.adv[b] = jdone;
    if (p.rej) p.rej[b] = jr >= 0 ? 1 : 0;
    for (int j = jdone; j < p.K; ++j) {
      if (p.logratio) p.logratio[static_cast<int64_t>(b) * p.K + j] = 0.f;
      if (p.logu) p.logu[static_cast<int64_t>(b) * p.K + j] = 0.f;
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (own[e]) p.x_out[static_cast<int64_t>(b) * d + 4 * gl + e] = static_cast<float>(cur[e]);
}

// Windows back to back for the chains of a wavefront (sd_langevin_run_phi4).  A chain's walk is a sequence of
// steps, each of which costs one gradient at its current state and one draw of noise, whether the step opens a
// window (the gradient is the frozen one and the position is accepted by construction) or tests a draft (the
// gradient gives Delta).  So the 64 / G chains of a wavefront stay in lockstep step by step although their
// windows start and end at different times, and no lane idles before its chain has reached T.
// Noise and uniforms are keyed by chain and absolute step, so the values are those of the window kernel;
// the uniforms are drawn G steps at a time and the batch carries over from one window to the next.  At the end
// of a window the state passes through fp32, as it does between sd_langevin_window_phi4 and the next call:
// the result is bit for bit that of window + advance repeated.
template <int G>
__global__ __launch_bounds__(256) void phi4_run_kernel(Phi4Args p) {
  constexpr int CPWV = 64 / G;
  extern __shared__ __align__(16) double sh_x[];     // [256 / G][d]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int sub = lane / G, gl = lane % G;
  const int slot = wave * CPWV + sub;
  const int Bact = p.active ? min(p.B, max(0, *p.active)) : p.B;
  const int b_raw = blockIdx.x * (4 * CPWV) + slot;
  const bool valid = b_raw < Bact;
  const int b = valid ? b_raw : 0;
  const int d = p.d, L = p.L;
  int n = valid ? p.n[b] : p.T;
  const int64_t id = valid ? p.id[b] : 0;
  const double gamma = p.gamma, beta2 = 2.0 * p.beta;
  const double sq2g = sqrt(2.0 * gamma), sqg2 = sqrt(0.5 * gamma), inv_sqg2 = 1.0 / sqg2;
  double* xs = sh_x + static_cast<size_t>(slot) * d;

  bool own[4];
  int nb[4][4];
  double cur[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int s = 4 * gl + e;
    own[e] = s < d;
    const int sc = own[e] ? s : 0;
    const int r = sc / L, c = sc % L;
    nb[e][0] = ((r + L - 1) % L) * L + c;
    nb[e][1] = ((r + 1) % L) * L + c;
    nb[e][2] = r * L + (c + L - 1) % L;
    nb[e][3] = r * L + (c + 1) % L;
    cur[e] = (valid && own[e]) ? static_cast<double>(p.x[static_cast<int64_t>(b) * d + s]) : 0.0;
  }

  auto gradient = [&](double g[4]) {               // as in phi4_window_kernel: every lane of the wavefront takes part
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (own[e]) xs[4 * gl + e] = cur[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      double v = 0.0;
      if (own[e]) {
        const double s4 = xs[nb[e][0]] + xs[nb[e][1]] + xs[nb[e][2]] + xs[nb[e][3]];
        v = beta2 * (4.0 * cur[e] - s4) + 4.0 * cur[e] * (cur[e] * cur[e] - 1.0);
      }
      g[e] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };

  int Kt = max(0, min(p.K, p.T - n));
  int j = 0, windows = 0;
  bool active = valid && Kt > 0;
  double g0[4] = {0.0, 0.0, 0.0, 0.0};
  int lu_base = 0;                                   // first absolute step of the batch of uniforms held in lu_batch
  bool lu_have = false;
  double lu_batch = 0.0;
  unsigned long long acc_adv = 0, acc_win = 0, acc_rej = 0, acc_kt = 0;

  // Ends: a step moves every active chain forward by one position, a window of Kt positions ends after at
  // most Kt steps and advances n by at least 1, and a chain stops at n = T or after max_windows windows.
  while (__ballot(active) != 0ull) {
    double g[4];
    gradient(g);
    if (active) {                                    // the lanes of a chain agree
      const int k1 = n + j + 1;                      // absolute step this position produces
      float z[4];
      sdrng::normal4(p.seed, id, static_cast<uint32_t>(k1), sdrng::kStreamNoise, static_cast<uint32_t>(gl), z);
      bool ended = false, rejected = false;
      if (j == 0) {                                  // window start: this gradient is the frozen one
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          g0[e] = g[e];
          if (own[e]) cur[e] = cur[e] - gamma * g0[e] + sq2g * static_cast<double>(z[e]);
        }
      } else {
        if (!lu_have || k1 - lu_base >= G) {
          lu_base = k1;
          lu_have = true;
          lu_batch = sdrng::log_uniform(p.seed, id, static_cast<uint32_t>(k1 + gl));
        }
        const double lu = __shfl(lu_batch, sub * G + (k1 - lu_base), 64);
        double dl[4], a1 = 0.0, a2 = 0.0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dl[e] = own[e] ? sqg2 * (g[e] - g0[e]) : 0.0;
          a1 = fma(static_cast<double>(z[e]), dl[e], a1);
          a2 = fma(dl[e], dl[e], a2);
        }
        const double S1 = group_sum_f64<G>(a1), S2 = group_sum_f64<G>(a2);
        const double lr = (-S1 - 0.5 * S2) * p.inv_tau;
        rejected = !(S2 == 0.0 || (lr == lr && lu <= fmin(0.0, lr)));
        const double coef = S2 > 0.0 ? S1 / S2 : 0.0;
        if (rejected) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (own[e])
              cur[e] = cur[e] - gamma * (g0[e] + dl[e] * inv_sqg2) + sq2g * (static_cast<double>(z[e]) - 2.0 * coef * dl[e]);
          ended = true;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (own[e]) cur[e] = cur[e] - gamma * g0[e] + sq2g * static_cast<double>(z[e]);
        }
      }
      ++j;
      if (j == Kt) ended = true;
      if (ended) {
        n += j;
        acc_adv += j; acc_win += 1; acc_rej += rejected ? 1 : 0; acc_kt += Kt;
#pragma unroll
        for (int e = 0; e < 4; ++e) cur[e] = static_cast<double>(static_cast<float>(cur[e]));
        ++windows;
        j = 0;
        Kt = max(0, min(p.K, p.T - n));
        active = Kt > 0 && windows < p.max_windows;
      }
    }
  }

  if (!valid) return;
  if (gl == 0) {
    p.n_out[b] = n;
    if (p.counters && acc_win) {
      atomicAdd(&p.counters[0], acc_adv);
      atomicAdd(&p.counters[1], acc_win);
      atomicAdd(&p.counters[2], acc_rej);
      atomicAdd(&p.counters[4], acc_kt);
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (own[e]) p.x_out[static_cast<int64_t>(b) * d + 4 * gl + e] = static_cast<float>(cur[e]);
}

template <int G>
hipError_t launch_phi4_run(const Phi4Args& p, hipStream_t st) {
  constexpr int chains_per_wg = 256 / G;
  const size_t shmem = sizeof(double) * static_cast<size_t>(chains_per_wg) * p.d;
  const unsigned grid = static_cast<unsigned>((p.B + chains_per_wg - 1) / chains_per_wg);
  hipLaunchKernelGGL(phi4_run_kernel<G>, dim3(grid), dim3(256), shmem, st, p);
  return hipGetLastError();
}

template <int G>
hipError_t launch_phi4(const Phi4Args& p, hipStream_t st) {
  constexpr int chains_per_wg = 256 / G;
  const size_t shmem = sizeof(double) * static_cast<size_t>(chains_per_wg) * p.d;
  const unsigned grid = static_cast<unsigned>((p.B + chains_per_wg - 1) / chains_per_wg);
  hipLaunchKernelGGL(phi4_window_kernel<G>, dim3(grid), dim3(256), shmem, st, p);
  return hipGetLastError();
}

}  // namespace

// One-time set-up on the current device, called by sd_create: dynamic-LDS limits of every instantiation of the
// wavefront kernel (so that no launch path carries set-up calls or "already done" flags) and the CU count.
hipError_t sdi::langevin_prepare(int* cus) {
  hipError_t e = hipSuccess;
#define SD_PREP(c_) \
  if (e == hipSuccess) e = prepare_wave<c_, false, false>(); \
  if (e == hipSuccess) e = prepare_wave<c_, false, true>();  \
  if (e == hipSuccess) e = prepare_wave<c_, true, false>();  \
  if (e == hipSuccess) e = prepare_wave<c_, true, true>();
  SD_PREP(1) SD_PREP(2) SD_PREP(3) SD_PREP(4)
#undef SD_PREP
  int dev = 0, n = 0;
  if (e == hipSuccess) e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
  *cus = n > 0 ? n : 256;
  return e;
}

namespace {

// Shared by sd_langevin_window (max_windows = 1) and sd_langevin_run.
int langevin_launch(const char* who, sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                    const int64_t* chain_id, const float* means, const float* logw, float comp_std, int32_t M,
                    float gamma, float* x_out, int32_t* adv, uint8_t* rejected, float* logratio, float* logu,
                    int32_t max_windows, int32_t* n_out, int64_t* counters, void* stream) {
  if (M > 16)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "%s: at most 16 mixture components (M=%d)", who, M);
  const int groups = (ctx->d + 3) / 4;
  const int cpt = (groups + kThreads - 1) / kThreads;
  if (cpt > 4)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "%s: d=%d exceeds the register-resident limit of %d", who,
                     ctx->d, 4 * 4 * kThreads);
  LangevinArgs p;
  p.x = x; p.n = n; p.id = chain_id; p.means = means; p.logw = logw; p.x_out = x_out; p.adv = adv;
  p.rej = rejected; p.logratio = logratio; p.logu = logu; p.active = ctx->active; p.queue = ctx->dev_queue;
  p.B = B; p.d = ctx->d; p.K = ctx->K; p.T = ctx->T; p.M = M; p.seed = ctx->seed;
  p.gamma = gamma; p.inv_s2 = 1.0 / (static_cast<double>(comp_std) * comp_std); p.inv_tau = 1.0 / ctx->tau;
  p.max_windows = max_windows; p.n_out = n_out; p.counters = reinterpret_cast<unsigned long long*>(counters);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int dpad = 4 * groups;
  if (dpad <= 1024) {                       // a wavefront per chain, means in LDS (16 rows of doubles, <= 128 KiB)
    hipError_t e;
    const bool whole = ctx->d % 4 == 0;
    const int sel = ((groups + 63) / 64 - 1) * 4 + (whole ? 2 : 0) + (max_windows > 1 ? 1 : 0);
    switch (sel) {
      case 0: e = launch_wave<1, false, false>(p, dpad, ctx->cus, st); break;
      case 1: e = launch_wave<1, false, true>(p, dpad, ctx->cus, st); break;
      case 2: e = launch_wave<1, true, false>(p, dpad, ctx->cus, st); break;
      case 3: e = launch_wave<1, true, true>(p, dpad, ctx->cus, st); break;
      case 4: e = launch_wave<2, false, false>(p, dpad, ctx->cus, st); break;
      case 5: e = launch_wave<2, false, true>(p, dpad, ctx->cus, st); break;
      case 6: e = launch_wave<2, true, false>(p, dpad, ctx->cus, st); break;
      case 7: e = launch_wave<2, true, true>(p, dpad, ctx->cus, st); break;
      case 8: e = launch_wave<3, false, false>(p, dpad, ctx->cus, st); break;
      case 9: e = launch_wave<3, false, true>(p, dpad, ctx->cus, st); break;
      case 10: e = launch_wave<3, true, false>(p, dpad, ctx->cus, st); break;
      case 11: e = launch_wave<3, true, true>(p, dpad, ctx->cus, st); break;
      case 12: e = launch_wave<4, false, false>(p, dpad, ctx->cus, st); break;
      case 13: e = launch_wave<4, false, true>(p, dpad, ctx->cus, st); break;
      case 14: e = launch_wave<4, true, false>(p, dpad, ctx->cus, st); break;
      default: e = launch_wave<4, true, true>(p, dpad, ctx->cus, st); break;
    }
    if (e != hipSuccess) return sdi::fail(ctx->err, SD_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
    if (max_windows > 1 && counters) hipLaunchKernelGGL(bump_launches_kernel, dim3(1), dim3(1), 0, st, p.counters);
    return SD_OK;
  }
  if (max_windows > 1)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "%s: d=%d is above the 1024 the back-to-back form serves", who, ctx->d);
  const dim3 grid(static_cast<unsigned>(B)), block(kThreads);
  switch (cpt) {
    case 1: hipLaunchKernelGGL((langevin_window_kernel<1, 16>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((langevin_window_kernel<2, 16>), grid, block, 0, st, p); break;
    default: hipLaunchKernelGGL((langevin_window_kernel<4, 16>), grid, block, 0, st, p); break;
  }
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

}  // namespace

extern "C" int sd_langevin_window(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                                  const int64_t* chain_id, const float* means, const float* logw,
                                  float comp_std, int32_t M, float gamma, float* x_out, int32_t* adv,
                                  uint8_t* rejected, float* logratio, float* logu, void* stream) {
  if (!ctx) return SD_ERR_ARG;
  if (B < 0 || M <= 0 || !(comp_std > 0.f) || !(gamma > 0.f) ||
      (B > 0 && (!x || !n || !chain_id || !means || !logw || !x_out || !adv)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_langevin_window: bad argument");
  if (B == 0) return SD_OK;
  return langevin_launch("sd_langevin_window", ctx, B, x, n, chain_id, means, logw, comp_std, M, gamma, x_out, adv,
                         rejected, logratio, logu, 1, nullptr, nullptr, stream);
}

extern "C" int sd_langevin_run(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n, const int64_t* chain_id,
                               const float* means, const float* logw, float comp_std, int32_t M, float gamma,
                               int32_t max_windows, float* x_out, int32_t* n_out, int64_t* counters, void* stream) {
  if (!ctx) return SD_ERR_ARG;
  if (B < 0 || M <= 0 || !(comp_std > 0.f) || !(gamma > 0.f) || max_windows < 2 ||
      (B > 0 && (!x || !n || !chain_id || !means || !logw || !x_out || !n_out)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_langevin_run: bad argument (max_windows >= 2)");
  if (B == 0) return SD_OK;
  return langevin_launch("sd_langevin_run", ctx, B, x, n, chain_id, means, logw, comp_std, M, gamma, x_out, nullptr,
                         nullptr, nullptr, nullptr, max_windows, n_out, counters, stream);
}

extern "C" int sd_langevin_window_phi4(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                                       const int64_t* chain_id, int32_t L, float beta, float gamma, float* x_out,
                                       int32_t* adv, uint8_t* rejected, float* logratio, float* logu, void* stream) {
  if (!ctx) return SD_ERR_ARG;
  if (B < 0 || L < 3 || !(beta >= 0.f) || !(gamma > 0.f) || (B > 0 && (!x || !n || !chain_id || !x_out || !adv)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_langevin_window_phi4: bad argument (L >= 3, beta >= 0, gamma > 0)");
  if (L * L != ctx->d)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_langevin_window_phi4: the context's d=%d is not L*L=%d", ctx->d, L * L);
  if (ctx->d > 256)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_langevin_window_phi4: grids up to 16 x 16 (d=%d)", ctx->d);
  if (B == 0) return SD_OK;
  Phi4Args p;
  p.x = x; p.n = n; p.id = chain_id; p.x_out = x_out; p.adv = adv; p.rej = rejected; p.logratio = logratio; p.logu = logu;
  p.active = ctx->active; p.B = B; p.d = ctx->d; p.L = L; p.K = ctx->K; p.T = ctx->T; p.seed = ctx->seed;
  p.gamma = gamma; p.beta = beta; p.inv_tau = 1.0 / ctx->tau;
  p.max_windows = 1; p.n_out = nullptr; p.counters = nullptr;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int groups = (ctx->d + 3) / 4;
  hipError_t e;
  if (groups <= 4) e = launch_phi4<4>(p, st);
  else if (groups <= 8) e = launch_phi4<8>(p, st);
  else if (groups <= 16) e = launch_phi4<16>(p, st);
  else if (groups <= 32) e = launch_phi4<32>(p, st);
  else e = launch_phi4<64>(p, st);
  if (e != hipSuccess) return sdi::fail(ctx->err, SD_ERR_HIP, "sd_langevin_window_phi4: %s", hipGetErrorString(e));
  return SD_OK;
}

extern "C" int sd_langevin_run_phi4(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n, const int64_t* chain_id,
                                    int32_t L, float beta, float gamma, int32_t max_windows, float* x_out,
                                    int32_t* n_out, int64_t* counters, void* stream) {
  if (!ctx) return SD_ERR_ARG;
  if (B < 0 || L < 3 || !(beta >= 0.f) || !(gamma > 0.f) || max_windows < 2 ||
      (B > 0 && (!x || !n || !chain_id || !x_out || !n_out)))
    return sdi::fail(ctx->err, SD_ERR_ARG,
                     "sd_langevin_run_phi4: bad argument (L >= 3, beta >= 0, gamma > 0, max_windows >= 2)");
  if (L * L != ctx->d)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_langevin_run_phi4: the context's d=%d is not L*L=%d", ctx->d, L * L);
  if (ctx->d > 256)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_langevin_run_phi4: grids up to 16 x 16 (d=%d)", ctx->d);
  if (B == 0) return SD_OK;
  Phi4Args p;
  p.x = x; p.n = n; p.id = chain_id; p.x_out = x_out; p.adv = nullptr; p.rej = nullptr; p.logratio = nullptr; p.logu = nullptr;
  p.active = ctx->active; p.B = B; p.d = ctx->d; p.L = L; p.K = ctx->K; p.T = ctx->T; p.seed = ctx->seed;
  p.gamma = gamma; p.beta = beta; p.inv_tau = 1.0 / ctx->tau;
  p.max_windows = max_windows; p.n_out = n_out; p.counters = reinterpret_cast<unsigned long long*>(counters);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int groups = (ctx->d + 3) / 4;
  hipError_t e;
  if (groups <= 4) e = launch_phi4_run<4>(p, st);
  else if (groups <= 8) e = launch_phi4_run<8>(p, st);
  else if (groups <= 16) e = launch_phi4_run<16>(p, st);
  else if (groups <= 32) e = launch_phi4_run<32>(p, st);
  else e = launch_phi4_run<64>(p, st);
  if (e != hipSuccess) return sdi::fail(ctx->err, SD_ERR_HIP, "sd_langevin_run_phi4: %s", hipGetErrorString(e));
  if (counters) hipLaunchKernelGGL(bump_launches_kernel, dim3(1), dim3(1), 0, st, p.counters);
  return SD_OK;
}
