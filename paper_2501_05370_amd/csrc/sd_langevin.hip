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
// One workgroup per chain.  A thread owns CPT groups of four consecutive coordinates (= one
// Philox block each), keeps the window state, the frozen gradient and its slice of the mixture
// means in registers, and walks the window positions in order; because the whole chain lives in
// one workgroup the walk simply stops at the first rejection, so no work is spent on drafts
// that would be discarded.  Per position: 16 logit partial sums and the two dot products are
// reduced over the workgroup in fp64.
#include <hip/hip_runtime.h>

#include <cmath>

#include "sd_internal.h"
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
  int B, d, K, T, M;
  uint64_t seed;
  double gamma, inv_s2, inv_tau;
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
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
      for (int s = 32; s >= 1; s >>= 1) mx = fmax(mx, __shfl_xor(mx, s, 64));
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
      reject = !(S2 == 0.0 || lu <= fmin(0.0, lr));
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
  if (M > 16)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_langevin_window: at most 16 mixture components (M=%d)", M);
  const int groups = (ctx->d + 3) / 4;
  const int cpt = (groups + kThreads - 1) / kThreads;
  if (cpt > 4)
    return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_langevin_window: d=%d exceeds the register-resident limit of %d",
                     ctx->d, 4 * 4 * kThreads);
  LangevinArgs p;
  p.x = x; p.n = n; p.id = chain_id; p.means = means; p.logw = logw; p.x_out = x_out; p.adv = adv;
  p.rej = rejected; p.logratio = logratio; p.logu = logu; p.active = ctx->active;
  p.B = B; p.d = ctx->d; p.K = ctx->K; p.T = ctx->T; p.M = M; p.seed = ctx->seed;
  p.gamma = gamma; p.inv_s2 = 1.0 / (static_cast<double>(comp_std) * comp_std); p.inv_tau = 1.0 / ctx->tau;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(static_cast<unsigned>(B)), block(kThreads);
  switch (cpt) {
    case 1: hipLaunchKernelGGL((langevin_window_kernel<1, 16>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((langevin_window_kernel<2, 16>), grid, block, 0, st, p); break;
    default: hipLaunchKernelGGL((langevin_window_kernel<4, 16>), grid, block, 0, st, p); break;
  }
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}
