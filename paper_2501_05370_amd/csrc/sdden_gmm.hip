// Posterior mean of a diagonal-covariance Gaussian mixture under the forward noising
// x_t = sqrt(ab) x0 + sqrt(1-ab) eps -- the analytic stand-in for the target network
// (paper Sec. 3.1 treats the drift as a black box; the low-dimensional mixture study of the
// experiments has this shape).  Also the generic entry points of sdden.h.
//
//   r_m(x)  = softmax_m( log w_m + log N(x; sqrt(ab) mu_m, diag(ab s_m^2 + 1-ab)) )
//   D(x,k)  = sum_m r_m(x) ( mu_m + sqrt(ab) s_m^2 / v_m * (x - sqrt(ab) mu_m) )
//
// One wavefront per row.  Phase 1: a lane owns a component and walks the coordinates (no
// cross-lane reduction for the logits).  Phase 2: a lane owns a coordinate and walks the
// components.  All arithmetic in fp64: the rows are few and small, and the responsibilities are
// exponentials of sums of d terms.  Reciprocal variances use the fp32 hardware reciprocal refined by
// two Newton steps in fp64 (relative error ~1e-14) instead of full fp64 divisions.
#include <cmath>
#include <new>
#include <vector>

#include "sd_lanes.h"
#include "sdden_internal.h"

namespace sdi {
std::string g_den_create_error;
}

namespace {

constexpr int kRowsPerBlock = 4;

constexpr int kRegNI = 32;   // coordinates per lane of the register-resident kernel

struct GmmArgs {
  const float* X;
  const int32_t* krow;
  float* out;
  const float *mu, *sd;      // [M,d]  component means and stds
  const float *muT, *sdT;    // [d,M]  the same, transposed
  const float2* lane_tab;    // [kRegNI,64] (mean, std) in the lane order of the register kernel, or null
  const double* cst;         // [T,M]  log w_m - 1/2 sum_i log v_mi(k)
  int Mp;                    // M rounded up to a power of two (<= 64), lanes per coordinate slice
  const float* ab;           // [T+1]
  const int32_t* active;
  int rows_per_chain;
  int R, d, M, T;
};

// 1/v for v in [~1e-3, ~1e3]: the hardware fp32 reciprocal (1 ulp; the correctly rounded one is a
// ten-instruction sequence), then y <- y (2 - v y) twice.
__device__ __forceinline__ double reciprocal(double v) {
  double y = static_cast<double>(__builtin_amdgcn_rcpf(static_cast<float>(v)));
  y = y * fma(-v, y, 2.0);
  y = y * fma(-v, y, 2.0);
  return y;
}

// One Newton step: relative error < 4e-14 (the start is within 2e-7), far inside the 1e-5 of the parity contract.
__device__ __forceinline__ double reciprocal_one_step(double v) {
  const double y = static_cast<double>(__builtin_amdgcn_rcpf(static_cast<float>(v)));
  return y * fma(-v, y, 2.0);
}

__global__ __launch_bounds__(64 * kRowsPerBlock) void gmm_posterior_mean_kernel(GmmArgs p) {
  extern __shared__ double smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  double* rs = smem + static_cast<size_t>(wave) * (p.M + p.d);   // [M] responsibilities
  double* xs = rs + p.M;                                          // [d] the row
  const int r = blockIdx.x * kRowsPerBlock + wave;
  const int Ract = sdi::active_rows(p.active, p.rows_per_chain, p.R);
  const int k = r < Ract ? p.krow[r] : -1;
  // masked row (k < 0) or a step the chain does not have; the whole wavefront leaves together, no barriers used
  if (static_cast<unsigned>(k) >= static_cast<unsigned>(p.T)) return;
  const double ab = p.ab[k];
  const double sab = sqrt(ab), om = 1.0 - ab;
  const float* x = p.X + static_cast<int64_t>(r) * p.d;
  for (int i = lane; i < p.d; i += 64) xs[i] = x[i];
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();

  double mx = -INFINITY;
  if (p.Mp < 64) {
    // fewer than 64 components: 64/Mp lanes share a component and split the coordinates
    const int m = lane % p.Mp, part = lane / p.Mp, parts = 64 / p.Mp;
    double q = 0.0;
    if (m < p.M) {
      for (int i = part; i < p.d; i += parts) {
        const double diff = xs[i] - sab * p.muT[static_cast<int64_t>(i) * p.M + m];
        const double sd = p.sdT[static_cast<int64_t>(i) * p.M + m];
        const double iv = reciprocal(ab * sd * sd + om);
        q = fma(diff * diff, iv, q);
      }
    }
    for (int s = p.Mp; s < 64; s <<= 1) q += __shfl_xor(q, s, 64);
    if (m < p.M && part == 0) {
      const double logit = p.cst[static_cast<int64_t>(k) * p.M + m] - 0.5 * q;
      rs[m] = logit;
      mx = logit;
    }
  } else {
    for (int m = lane; m < p.M; m += 64) {
      double q = 0.0;
      for (int i = 0; i < p.d; ++i) {
        const double diff = xs[i] - sab * p.muT[static_cast<int64_t>(i) * p.M + m];
        const double sd = p.sdT[static_cast<int64_t>(i) * p.M + m];
        const double iv = reciprocal(ab * sd * sd + om);
        q = fma(diff * diff, iv, q);
      }
      const double logit = p.cst[static_cast<int64_t>(k) * p.M + m] - 0.5 * q;
      rs[m] = logit;
      mx = fmax(mx, logit);
    }
  }
  for (int s = 32; s >= 1; s >>= 1) mx = fmax(mx, __shfl_xor(mx, s, 64));
  double sum = 0.0;
  for (int m = lane; m < p.M; m += 64) {
    const double e = exp(rs[m] - mx);
    rs[m] = e;
    sum += e;
  }
  for (int s = 32; s >= 1; s >>= 1) sum += __shfl_xor(sum, s, 64);
  const double inv = 1.0 / sum;
  __builtin_amdgcn_wave_barrier();
  __threadfence_block();

  float* o = p.out + static_cast<int64_t>(r) * p.d;
  for (int i = lane; i < p.d; i += 64) {
    const double xi = xs[i];
    double acc = 0.0;
    for (int m = 0; m < p.M; ++m) {
      if (rs[m] < 1e-25) continue;          // the same for every lane; such a component moves nothing
      const double mu = p.mu[static_cast<int64_t>(m) * p.d + i];
      const double sd = p.sd[static_cast<int64_t>(m) * p.d + i];
      const double s2 = sd * sd;
      const double iv = reciprocal(ab * s2 + om);
      acc += rs[m] * (mu + sab * s2 * iv * (xi - sab * mu));
    }
    o[i] = static_cast<float>(acc * inv);
  }
}

// Small mixtures (MP = M rounded up to a power of two <= 32, d <= (64 / MP) * NI): a lane computes the
// per-component posterior mean of its (component, coordinate) pairs in the same pass as the quadratic
// form and keeps it in registers, so the reciprocal variance and x - sqrt(ab) mu are computed once
// instead of once per phase.
// Lane = part + PARTS * m (component m, PARTS = 64 / MP lanes per component); the lane owns coordinates
// i = part + PARTS * j, j < NI.  Phase 1 sums its quadratic form and finishes it across the parts; the
// softmax runs across the component lanes; phase 2 scales the kept means by r_m and a halving exchange over
// the component lanes leaves each lane with the finished sums of NI / MP coordinates, which it writes.
// The component index sits in the high lane bits so that the two largest levels of the exchange (half
// and a quarter of the list) are row swaps, one instruction per 32-bit word with no select.
// No LDS, no barrier.
__device__ __forceinline__ double lane_xor_f64(double v, int mask) {   // mask: one bit, constant after unrolling
  switch (mask) {
    case 1: return sdlane::lane_xor<1>(v);
    case 2: return sdlane::lane_xor<2>(v);
    case 4: return sdlane::lane_xor<4>(v);
    case 8: return sdlane::lane_xor<8>(v);
    case 16: return sdlane::lane_xor<16>(v);
    default: return sdlane::lane_xor<32>(v);
  }
}

__device__ __forceinline__ double halving_add_f64(double lower, double upper, int mask) {
  switch (mask) {
    case 1: return sdlane::halving_add<1>(lower, upper);
    case 2: return sdlane::halving_add<2>(lower, upper);
    case 4: return sdlane::halving_add<4>(lower, upper);
    case 8: return sdlane::halving_add<8>(lower, upper);
    case 16: return sdlane::halving_add<16>(lower, upper);
    default: return sdlane::halving_add<32>(lower, upper);
  }
}

template <int MP, int NI>
__global__ __launch_bounds__(64 * kRowsPerBlock) void gmm_posterior_mean_reg_kernel(GmmArgs p) {
  static_assert(NI % MP == 0 && MP <= 32 && (MP & (MP - 1)) == 0, "component lanes must divide the coordinate list");
  constexpr int PARTS = 64 / MP;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = blockIdx.x * kRowsPerBlock + wave;
  const int Ract = sdi::active_rows(p.active, p.rows_per_chain, p.R);
  const int k = r < Ract ? p.krow[r] : -1;
  // masked row (k < 0) or a step the chain does not have; the whole wavefront leaves together
  if (static_cast<unsigned>(k) >= static_cast<unsigned>(p.T)) return;
  const double ab = p.ab[k];
  const double sab = sqrt(ab), om = 1.0 - ab;
  const int part = lane % PARTS, m = lane / PARTS;
  const bool live = m < p.M;
  const float* x = p.X + static_cast<int64_t>(r) * p.d;

  double v[NI];                             // posterior mean of component m at the owned coordinates
  double q = 0.0;
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int i = part + PARTS * j;
    v[j] = 0.0;
    if (live && i < p.d) {
      const float2 ms = p.lane_tab[j * 64 + lane];           // one coalesced 512-byte read per wavefront
      const double mu = ms.x, sd = ms.y;
      const double s2 = sd * sd;
      const double iv = reciprocal_one_step(fma(ab, s2, om));
      const double df = fma(-sab, mu, static_cast<double>(x[i]));
      q = fma(df * df, iv, q);
      v[j] = fma(sab * s2 * iv, df, mu);
    }
  }
#pragma unroll
  for (int s = 1; s < PARTS; s <<= 1) q += lane_xor_f64(q, s);
  const double logit = live ? p.cst[static_cast<int64_t>(k) * p.M + m] - 0.5 * q : -INFINITY;
  double mx = logit;
#pragma unroll
  for (int s = PARTS; s < 64; s <<= 1) mx = fmax(mx, lane_xor_f64(mx, s));
  const double e = live ? exp(logit - mx) : 0.0;
  double sum = e;
#pragma unroll
  for (int s = PARTS; s < 64; s <<= 1) sum += lane_xor_f64(sum, s);
  const double rm = e / sum;
#pragma unroll
  for (int j = 0; j < NI; ++j) v[j] *= rm;
  // halving exchange over the component lanes: at component distance s a lane keeps the upper half of its
  // list if bit s of its component is set (else the lower half) and adds the partner's sums for that half
  int n = NI;
#pragma unroll
  for (int s = MP / 2; s >= 1; s >>= 1) {
    n >>= 1;
#pragma unroll
    for (int j = 0; j < NI / 2; ++j)
      if (j < n) v[j] = halving_add_f64(v[j], v[j + n], s * PARTS);
  }
  constexpr int C = NI / MP;                // finished coordinates per lane: j = m * C + jj
  float* o = p.out + static_cast<int64_t>(r) * p.d;
#pragma unroll
  for (int jj = 0; jj < C; ++jj) {
    const int i = part + PARTS * (m * C + jj);
    if (i < p.d) o[i] = static_cast<float>(v[jj]);
  }
}

template <int MP, int NI>
void launch_reg(const GmmArgs& p, unsigned grid, hipStream_t st) {
  hipLaunchKernelGGL((gmm_posterior_mean_reg_kernel<MP, NI>), dim3(grid), dim3(64 * kRowsPerBlock), 0, st, p);
}

struct GmmDenoiser final : sdden {
  int M = 0, Mp = 1;          // Mp: M rounded up to a power of two, at most 64
  float* dev_f = nullptr;     // mu, sd, muT, sdT, ab, then the lane-ordered table when the register kernel applies
  const float2* lane_tab = nullptr;
  double* dev_cst = nullptr;
  ~GmmDenoiser() override {
    if (dev_f) (void)hipFree(dev_f);
    if (dev_cst) (void)hipFree(dev_cst);
  }
  int eval(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) override {
    GmmArgs p;
    const size_t md = static_cast<size_t>(M) * d;
    p.X = X; p.krow = krow; p.out = out;
    p.mu = dev_f; p.sd = dev_f + md; p.muT = dev_f + 2 * md; p.sdT = dev_f + 3 * md; p.ab = dev_f + 4 * md;
    p.Mp = Mp;
    p.lane_tab = lane_tab;
    p.cst = dev_cst; p.active = active; p.rows_per_chain = rows_per_chain;
    p.R = R; p.d = d; p.M = M; p.T = T;
    const size_t shmem = sizeof(double) * kRowsPerBlock * static_cast<size_t>(M + d);
    const unsigned grid = static_cast<unsigned>((R + kRowsPerBlock - 1) / kRowsPerBlock);
    prof.mark(1, st);
    if (lane_tab) {
      switch (p.Mp) {
        case 32: launch_reg<32, kRegNI>(p, grid, st); break;
        case 16: launch_reg<16, kRegNI>(p, grid, st); break;
        case 8: launch_reg<8, kRegNI>(p, grid, st); break;
        case 4: launch_reg<4, kRegNI>(p, grid, st); break;
        case 2: launch_reg<2, kRegNI>(p, grid, st); break;
        default: launch_reg<1, kRegNI>(p, grid, st); break;
      }
    } else {
      hipLaunchKernelGGL(gmm_posterior_mean_kernel, dim3(grid), dim3(64 * kRowsPerBlock), shmem, st, p);
    }
    prof.mark(1, st);
    SD_HIP_TRY(err, hipGetLastError());
    return SD_OK;
  }
};

}  // namespace

extern "C" {

int sdden_gmm_create(int32_t M, int32_t d, const float* means, const float* stds, const float* logw,
                     int32_t T, const float* alpha_bar_state, sdden** out) {
  std::string& E = sdi::g_den_create_error;
  if (!means || !stds || !logw || !alpha_bar_state || !out || M <= 0 || d <= 0 || T <= 0)
    return sdi::fail(E, SD_ERR_ARG, "sdden_gmm_create: bad argument");
  if (static_cast<size_t>(M + d) * sizeof(double) * kRowsPerBlock > 60000)
    return sdi::fail(E, SD_ERR_UNSUPPORTED, "sdden_gmm_create: M+d=%d too large for the LDS staging", M + d);
  const size_t md = static_cast<size_t>(M) * d;
  std::vector<float> h(4 * md + T + 1);
  std::vector<double> cst(static_cast<size_t>(T) * M);
  for (int m = 0; m < M; ++m)
    for (int i = 0; i < d; ++i) {
      const float mu = means[m * static_cast<size_t>(d) + i], s = stds[m * static_cast<size_t>(d) + i];
      if (!(s > 0.f)) return sdi::fail(E, SD_ERR_ARG, "sdden_gmm_create: stds must be > 0");
      h[m * static_cast<size_t>(d) + i] = mu;
      h[md + m * static_cast<size_t>(d) + i] = s;
      h[2 * md + i * static_cast<size_t>(M) + m] = mu;
      h[3 * md + i * static_cast<size_t>(M) + m] = s;
    }
  for (int k = 0; k <= T; ++k) h[4 * md + k] = alpha_bar_state[k];
  int Mp = 1;
  while (Mp < M && Mp < 64) Mp <<= 1;
  size_t lane_off = 0;
  if (Mp <= 32 && d <= (64 / Mp) * kRegNI) {
    // (mean, std) of the pair that lane part + PARTS * m reads at its j-th coordinate i = part + PARTS * j;
    // slots without a pair hold (0, 1) and are never used
    const int parts = 64 / Mp;
    lane_off = (h.size() + 1) / 2 * 2;                       // 8-byte aligned
    h.resize(lane_off + 2 * static_cast<size_t>(kRegNI) * 64);
    for (int j = 0; j < kRegNI; ++j)
      for (int lane = 0; lane < 64; ++lane) {
        const int part = lane % parts, m = lane / parts, i = part + parts * j;
        const bool has = m < M && i < d;
        h[lane_off + 2 * (static_cast<size_t>(j) * 64 + lane)] = has ? means[m * static_cast<size_t>(d) + i] : 0.f;
        h[lane_off + 2 * (static_cast<size_t>(j) * 64 + lane) + 1] = has ? stds[m * static_cast<size_t>(d) + i] : 1.f;
      }
  }
  for (int k = 0; k < T; ++k) {
    const double ab = alpha_bar_state[k];
    for (int m = 0; m < M; ++m) {
      double ld = 0.0;
      for (int i = 0; i < d; ++i) {
        const double sd = h[md + m * static_cast<size_t>(d) + i];
        ld += std::log(ab * sd * sd + (1.0 - ab));
      }
      cst[static_cast<size_t>(k) * M + m] = static_cast<double>(logw[m]) - 0.5 * ld;
    }
  }
  GmmDenoiser* g = new (std::nothrow) GmmDenoiser;
  if (!g) return sdi::fail(E, SD_ERR_ARG, "sdden_gmm_create: out of host memory");
  g->d = d; g->T = T; g->M = M;
  hipError_t e = hipMalloc(&g->dev_f, h.size() * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&g->dev_cst, cst.size() * sizeof(double));
  if (e == hipSuccess) e = hipMemcpy(g->dev_f, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(g->dev_cst, cst.data(), cst.size() * sizeof(double), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    delete g;
    return sdi::fail(E, SD_ERR_HIP, "sdden_gmm_create: %s", hipGetErrorString(e));
  }
  g->Mp = Mp;
  if (lane_off) g->lane_tab = reinterpret_cast<const float2*>(g->dev_f + lane_off);
  *out = g;
  return SD_OK;
}

int sdden_eval(sdden* den, int32_t R, const float* X, const int32_t* krow, float* out, void* stream) {
  if (!den) return SD_ERR_ARG;
  if (R < 0 || (R > 0 && (!X || !krow || !out))) return sdi::fail(den->err, SD_ERR_ARG, "sdden_eval: bad argument");
  if (R == 0) return SD_OK;
  den->prof.cur_rows = R;
  return den->eval(R, X, krow, out, static_cast<hipStream_t>(stream));
}

int sdden_eval_mirror(sdden* den, int32_t R, const float* X, const uint16_t* Xbf16, const int32_t* krow, float* out,
                      void* stream) {
  if (!den) return SD_ERR_ARG;
  if (R < 0 || (R > 0 && (!X || !Xbf16 || !krow || !out)))
    return sdi::fail(den->err, SD_ERR_ARG, "sdden_eval_mirror: bad argument");
  if (R == 0) return SD_OK;
  den->prof.cur_rows = R;
  return den->eval_mirror(R, X, Xbf16, krow, out, static_cast<hipStream_t>(stream));
}

int sdden_reserve(sdden* den, int32_t Rmax) {
  if (!den) return SD_ERR_ARG;
  if (Rmax <= 0) return sdi::fail(den->err, SD_ERR_ARG, "sdden_reserve: Rmax must be > 0");
  return den->reserve(Rmax);
}

int sdden_profile(sdden* den, int32_t which) {
  if (!den || which < 0) return SD_ERR_ARG;
  den->prof.which = which;
  den->prof.used = 0;
  return SD_OK;
}

int sdden_profile_min_rows(sdden* den, int32_t min_rows) {
  if (!den || min_rows < 0) return SD_ERR_ARG;
  den->prof.min_rows = min_rows;
  return SD_OK;
}

int sdden_profile_collect(sdden* den, double* total_ms, int64_t* launches) {
  if (!den || !total_ms || !launches) return SD_ERR_ARG;
  sdden_profiler& pr = den->prof;
  double tot = 0.0;
  const size_t pairs = pr.used / 2;
  if (pairs) SD_HIP_TRY(den->err, hipEventSynchronize(pr.events[2 * pairs - 1]));
  for (size_t i = 0; i < pairs; ++i) {
    float ms = 0.f;
    SD_HIP_TRY(den->err, hipEventElapsedTime(&ms, pr.events[2 * i], pr.events[2 * i + 1]));
    tot += ms;
  }
  *total_ms = tot;
  *launches = static_cast<int64_t>(pairs);
  pr.used = 0;
  return SD_OK;
}

int sdden_set_active_count(sdden* den, const int32_t* count, int32_t rows_per_chain) {
  if (!den) return SD_ERR_ARG;
  if (count && rows_per_chain <= 0) return sdi::fail(den->err, SD_ERR_ARG, "sdden_set_active_count: rows_per_chain must be > 0");
  den->active = count;
  den->rows_per_chain = count ? rows_per_chain : 1;
  return SD_OK;
}

int sdden_destroy(sdden* den) {
  if (!den) return SD_ERR_ARG;
  delete den;
  return SD_OK;
}

const char* sdden_last_error(const sdden* den) {
  return den ? den->err.c_str() : sdi::g_den_create_error.c_str();
}

}  // extern "C"
