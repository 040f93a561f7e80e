// E[x0 | x_t] for x0 ~ N(mu, U U^T + s2 I): the closed-form linear denoiser of the image-shaped
// linear-Gaussian workload, evaluated for all rows of a batched target call with two skinny fp32
// MFMA GEMMs (paper: the target is queried on all drafted states of a window in one batch,
// Alg. "Speculative Sampling for DDM", (Par.) line).
//
// In the eigenbasis Q (d x r, orthonormal columns) of U U^T = Q diag(lam) Q^T the posterior-mean
// map G = sqrt(ab) S (ab S + (1-ab) I)^-1, S = U U^T + s2 I, is diagonal:
//   G = g_perp I + Q diag(g_i - g_perp) Q^T,  g_i = sqrt(ab)(lam_i+s2)/(ab(lam_i+s2)+1-ab),
//                                            g_perp = sqrt(ab) s2/(ab s2+1-ab),
//   D(x,k) = mu + G (x - sqrt(ab) mu)
//          = g_perp x + (1 - sqrt(ab) g_perp) mu + Q [ (g - g_perp) .* (Q^T x - sqrt(ab) Q^T mu) ].
// GEMM 1: P = X Q with the bracket applied per row in the epilogue (each row has its own step k);
// GEMM 2: out = P' Q^T + g_perp(k) x + (1 - sqrt(ab_k) g_perp(k)) mu.
//
// Kernels: for d a multiple of 32 the ring-buffered direct-to-LDS GEMM of lowrank_gemm.h (first
// product split over K into slabs that a small kernel adds and scales).  Other d fall back to the
// older kernel below: 128x128 / 64x128 output tile, K-step 16, 4 wavefronts (2x2) of
// v_mfma_f32_32x32x2f32 tiles, A stored transposed in LDS, global->register prefetch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "lowrank_gemm.h"
#include "sdden_internal.h"
#include "sdden_rows.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BN = 128, BK = 16, kThreads = 256;
constexpr int LDB = BN + 4;                    // LDS row stride of the B slice (floats)

struct GemmArgs {
  const float* A;        // [*, lda] row-major; row r of the tile problem is A[arow(r)]
  int lda;
  const float* Bm;       // [Kdim, N] row-major
  int N, Kdim;
  const int32_t* rowidx; // gathered rows, or nullptr: identity
  const int32_t* count;  // device: number of rows M
  int a_gather;          // 1: A rows are rowidx[r]; 0: A rows are r (dense intermediate)
  // epilogue data
  const int32_t* krow;   // chain step of source row
  const float* X;        // [*, d] original rows (stage 2)
  float* out;            // stage 1: P' [M, r] dense; stage 2: out [*, d] scattered to source rows
  const float *gain;     // [T, r]
  const float *sab, *gperp, *coef;   // [T]
  const float *qmu;      // [r]
  const float *mu;       // [d]
};

// BM: rows per workgroup tile (64 or 128).  The first GEMM has only r/128 column tiles, so for
// small row counts it uses 64-row tiles to put enough workgroups in flight.
template <int STAGE, int BM>
__global__ __launch_bounds__(kThreads) void lowrank_gemm_kernel(GemmArgs p) {
  constexpr int LDA = BM + 4;
  constexpr int TMI = BM / 64;                   // 32-row MFMA tiles per wavefront
  constexpr int ACH = BM / 64;                   // float4 loads of A per thread per K-step
  __shared__ float As[2][BK][LDA];
  __shared__ float Bs[2][BK][LDB];
  const int M = *p.count;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  if (tile_m * BM >= M) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // global -> LDS assignment: ACH float4 of A and two of B per thread per K-step
  int a_m[ACH], a_k4[ACH], b_k[2], b_n4[2];
  const float* a_src[ACH];
  bool b_ok[2];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int idx = t + kThreads * i;
    a_m[i] = idx >> 2; a_k4[i] = idx & 3;
    const int gm = tile_m * BM + a_m[i];
    const int r = gm < M ? gm : M - 1;                       // clamp: rows past M are never stored
    const int src = (p.a_gather && p.rowidx) ? p.rowidx[r] : r;
    a_src[i] = p.A + static_cast<int64_t>(src) * p.lda + 4 * a_k4[i];
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = t + kThreads * i;
    b_k[i] = idx >> 5; b_n4[i] = idx & 31;
    b_ok[i] = tile_n * BN + 4 * b_n4[i] < p.N;               // N is a multiple of 4
  }
  const float* b_src = p.Bm + tile_n * BN;

  f32x16 acc[TMI][2];
#pragma unroll
  for (int i = 0; i < TMI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  float4 ra[ACH], rb[2];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) ra[i] = *reinterpret_cast<const float4*>(a_src[i] + k0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      rb[i] = b_ok[i] ? *reinterpret_cast<const float4*>(b_src + static_cast<int64_t>(k0 + b_k[i]) * p.N + 4 * b_n4[i])
                      : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto stash = [&](int s) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      As[s][4 * a_k4[i] + 0][a_m[i]] = ra[i].x;
      As[s][4 * a_k4[i] + 1][a_m[i]] = ra[i].y;
      As[s][4 * a_k4[i] + 2][a_m[i]] = ra[i].z;
      As[s][4 * a_k4[i] + 3][a_m[i]] = ra[i].w;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) *reinterpret_cast<float4*>(&Bs[s][b_k[i]][4 * b_n4[i]]) = rb[i];
  };

  const int nk = p.Kdim / BK;                                // Kdim is a multiple of BK (checked on host)
  fetch(0);
  stash(0);
  __syncthreads();
  const int half = lane >> 5, l32 = lane & 31;
  for (int kt = 0; kt < nk; ++kt) {
    const int s = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * BK);
#pragma unroll
    for (int k = 0; k < BK; k += 2) {
      float a[TMI], b[2];
#pragma unroll
      for (int i = 0; i < TMI; ++i) a[i] = As[s][k + half][wm * (BM / 2) + i * 32 + l32];
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = Bs[s][k + half][wn * 64 + j * 32 + l32];
#pragma unroll
      for (int i = 0; i < TMI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) stash(s ^ 1);
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][v] is element (row = (v/4)*8 + half*4 + v%4, col = l32) of its 32x32 tile
#pragma unroll
  for (int i = 0; i < TMI; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gm = tile_m * BM + wm * (BM / 2) + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
      if (gm >= M) continue;
      const int src = p.rowidx ? p.rowidx[gm] : gm;
      const int k = p.krow[src];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int gn = tile_n * BN + wn * 64 + j * 32 + l32;
        if (gn >= p.N) continue;
        const float c = acc[i][j][v];
        if (STAGE == 1) {
          p.out[static_cast<int64_t>(gm) * p.N + gn] =
              p.gain[static_cast<int64_t>(k) * p.N + gn] * (c - p.sab[k] * p.qmu[gn]);
        } else {
          const int64_t o = static_cast<int64_t>(src) * p.N + gn;
          p.out[o] = c + p.gperp[k] * p.X[o] + p.coef[k] * p.mu[gn];
        }
      }
    }
  }
}

// Cyclic Jacobi eigen-decomposition of a symmetric n x n matrix (fp64, host).
// On return A's diagonal holds the eigenvalues and V's columns the eigenvectors.
void jacobi_eigen(std::vector<double>& A, std::vector<double>& V, int n) {
  V.assign(static_cast<size_t>(n) * n, 0.0);
  for (int i = 0; i < n; ++i) V[static_cast<size_t>(i) * n + i] = 1.0;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, diag = 0.0;
    for (int i = 0; i < n; ++i)
      for (int j = 0; j < n; ++j) (i == j ? diag : off) += A[static_cast<size_t>(i) * n + j] * A[static_cast<size_t>(i) * n + j];
    if (off <= 1e-30 * diag) break;
    for (int p = 0; p < n - 1; ++p)
      for (int q = p + 1; q < n; ++q) {
        const double apq = A[static_cast<size_t>(p) * n + q];
        if (apq == 0.0) continue;
        const double app = A[static_cast<size_t>(p) * n + p], aqq = A[static_cast<size_t>(q) * n + q];
        const double theta = (aqq - app) / (2.0 * apq);
        const double tt = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
        const double c = 1.0 / std::sqrt(tt * tt + 1.0), s = tt * c;
        for (int k = 0; k < n; ++k) {                       // columns p, q
          const double akp = A[static_cast<size_t>(k) * n + p], akq = A[static_cast<size_t>(k) * n + q];
          A[static_cast<size_t>(k) * n + p] = c * akp - s * akq;
          A[static_cast<size_t>(k) * n + q] = s * akp + c * akq;
        }
        for (int k = 0; k < n; ++k) {                       // rows p, q
          const double apk = A[static_cast<size_t>(p) * n + k], aqk = A[static_cast<size_t>(q) * n + k];
          A[static_cast<size_t>(p) * n + k] = c * apk - s * aqk;
          A[static_cast<size_t>(q) * n + k] = s * apk + c * aqk;
        }
        for (int k = 0; k < n; ++k) {
          const double vkp = V[static_cast<size_t>(k) * n + p], vkq = V[static_cast<size_t>(k) * n + q];
          V[static_cast<size_t>(k) * n + p] = c * vkp - s * vkq;
          V[static_cast<size_t>(k) * n + q] = s * vkp + c * vkq;
        }
      }
  }
}

struct LowRankDenoiser final : sdden {
  int eval_ring(int R, const float* X, const int32_t* krow, float* out, hipStream_t st);
  int r = 0, rpad = 0;          // rank, rank padded to a multiple of BK (extra columns are zero)
  float* dev = nullptr;         // all float tables in one allocation
  float *Q = nullptr, *QT = nullptr, *gain = nullptr, *sab = nullptr, *gperp = nullptr, *coef = nullptr,
        *qmu = nullptr, *mu = nullptr;
  // per-call scratch, sized by sdden_reserve
  int32_t* rowidx = nullptr;
  int32_t* count = nullptr;
  float* P = nullptr;
  float* part = nullptr;        // K-split partial sums of the first product
  lrgemm::RowInfo* rowinfo = nullptr;   // per compacted row: source row and the second product's per-row scalars
  int64_t part_rows = 0;
  int nsplit = 1;               // K split of the first product: fixed per denoiser, so that the order in which a
                                // prediction's terms are added never depends on how many rows a call carries
  int cap_rows = 0;

  ~LowRankDenoiser() override {
    if (dev) (void)hipFree(dev);
    if (rowidx) (void)hipFree(rowidx);
    if (count) (void)hipFree(count);
    if (P) (void)hipFree(P);
    if (part) (void)hipFree(part);
    if (rowinfo) (void)hipFree(rowinfo);
  }

  int reserve(int R) override {
    if (R <= cap_rows) return SD_OK;
    if (rowidx) (void)hipFree(rowidx);
    if (P) (void)hipFree(P);
    if (part) (void)hipFree(part);
    if (rowinfo) (void)hipFree(rowinfo);
    rowidx = nullptr; P = nullptr; part = nullptr; rowinfo = nullptr; cap_rows = 0; part_rows = 0;
    SD_HIP_TRY(err, hipMalloc(&rowidx, sizeof(int32_t) * static_cast<size_t>(R)));
    SD_HIP_TRY(err, hipMalloc(&P, sizeof(float) * static_cast<size_t>(R) * rpad));
    if (d % lrgemm::BK == 0) {
      const int64_t rows = static_cast<int64_t>(nsplit) * R;       // one slab of R rows per K range
      SD_HIP_TRY(err, hipMalloc(&part, sizeof(float) * static_cast<size_t>(rows) * rpad));
      part_rows = rows;
      SD_HIP_TRY(err, hipMalloc(&rowinfo, sizeof(lrgemm::RowInfo) * static_cast<size_t>(R)));
    }
    if (!count) SD_HIP_TRY(err, hipMalloc(&count, sizeof(int32_t)));
    cap_rows = R;
    return SD_OK;
  }

  int eval(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) override {
    if (!sdi::aligned16(X)) return sdi::fail(err, SD_ERR_ARG, "sdden_eval(lowrank): X must be 16-byte aligned");
    if (R > cap_rows)
      return sdi::fail(err, SD_ERR_WORKSPACE, "sdden_eval(lowrank): %d rows exceed the %d reserved (sdden_reserve)", R, cap_rows);
    hipLaunchKernelGGL(sdrows::compact_rows_kernel, dim3(sdrows::compact_rows_grid(R)), dim3(sdrows::kScan), 0, st, krow, rowidx, count,
                       active, rows_per_chain, R, T);
    if (part && sdi::aligned16(out)) return eval_ring(R, X, krow, out, st);     // 16-byte stores into out
    GemmArgs a;
    a.rowidx = rowidx; a.count = count; a.krow = krow; a.X = X;
    a.gain = gain; a.sab = sab; a.gperp = gperp; a.coef = coef; a.qmu = qmu; a.mu = mu;
    // stage 1: P' = gain .* (X Q - sab qmu)       [M, rpad]
    a.A = X; a.lda = d; a.Bm = Q; a.N = rpad; a.Kdim = d; a.a_gather = 1; a.out = P;
    prof.mark(1, st);
    if (R <= 4096)   // few rows (the window-start call): smaller tiles put more workgroups in flight
      hipLaunchKernelGGL((lowrank_gemm_kernel<1, 64>), dim3(((R + 63) / 64) * ((rpad + BN - 1) / BN)), dim3(kThreads), 0, st, a);
    else
      hipLaunchKernelGGL((lowrank_gemm_kernel<1, 128>), dim3(((R + 127) / 128) * ((rpad + BN - 1) / BN)), dim3(kThreads), 0, st, a);
    prof.mark(1, st);
    // stage 2: out = P' Q^T + gperp x + coef mu   [rows, d]
    a.A = P; a.lda = rpad; a.Bm = QT; a.N = d; a.Kdim = rpad; a.a_gather = 0; a.out = out;
    prof.mark(2, st);
    hipLaunchKernelGGL((lowrank_gemm_kernel<2, 128>), dim3(((R + 127) / 128) * ((d + BN - 1) / BN)), dim3(kThreads), 0, st, a);
    prof.mark(2, st);
    SD_HIP_TRY(err, hipGetLastError());
    return SD_OK;
  }
};

int LowRankDenoiser::eval_ring(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) {
  // first product: part_s = X[rowidx] Q (K range s), then P' = gain .* (sum_s part_s - sab qmu)
  // 64-row tiles: three workgroups fit a CU instead of two and the idle tail of the launch is shorter; over a pass
  // of the 3072-wide workload they take 6 % less time than 128-row tiles (the tile height changes no sum: same K
  // order per element).
  lrgemm::Args a{};
  a.A = X; a.arow = rowidx; a.lda = d; a.Bt = QT; a.ldb = d; a.N = rpad; a.Kdim = d; a.count = count;
  a.part = part; a.slab_stride = static_cast<int64_t>(R) * rpad;
  prof.mark(1, st);
  SD_HIP_TRY(err, (lrgemm::launch<64, 128, 1, 4, 1, 2>(a, R, nsplit, st)));
  prof.mark(1, st);
  const int64_t quads = static_cast<int64_t>(R) * (rpad / 4);
  hipLaunchKernelGGL(lrgemm::reduce_gain_kernel, dim3(static_cast<unsigned>((quads + 255) / 256)), dim3(256), 0, st, part,
                     a.slab_stride, nsplit, count, rowidx, krow, gain, sab, qmu, P, rpad, gperp, coef, rowinfo);
  // second product: out = P' Q^T + gperp x + coef mu
  lrgemm::Args b{};
  b.A = P; b.arow = nullptr; b.lda = rpad; b.Bt = Q; b.ldb = rpad; b.N = d; b.Kdim = rpad; b.count = count;
  b.rowinfo = rowinfo; b.X = X; b.out = out; b.mu = mu;
  prof.mark(2, st);
  SD_HIP_TRY(err, (lrgemm::launch<64, 128, 1, 4, 2, 2>(b, R, 1, st)));
  prof.mark(2, st);
  SD_HIP_TRY(err, hipGetLastError());
  return SD_OK;
}

}  // namespace

extern "C" int sdden_lowrank_create(int32_t d, int32_t r, const float* mu, const float* U, float s2, int32_t T,
                                    const float* alpha_bar_state, sdden** out) {
  std::string& E = sdi::g_den_create_error;
  if (!mu || !U || !alpha_bar_state || !out || d <= 0 || r <= 0 || T <= 0 || !(s2 > 0.f))
    return sdi::fail(E, SD_ERR_ARG, "sdden_lowrank_create: bad argument");
  if (d % BK != 0)
    return sdi::fail(E, SD_ERR_UNSUPPORTED, "sdden_lowrank_create: d=%d must be a multiple of %d", d, BK);
  const int rpad = ((r + lrgemm::BK - 1) / lrgemm::BK) * lrgemm::BK;     // multiple of both kernels' K-steps
  // Gram matrix G = U^T U (r x r), its eigen-decomposition, and Q = U V diag(lam^-1/2)
  std::vector<double> G(static_cast<size_t>(r) * r, 0.0), V;
  for (int i = 0; i < d; ++i) {
    const float* row = U + static_cast<size_t>(i) * r;
    for (int a = 0; a < r; ++a) {
      const double ua = row[a];
      for (int b = a; b < r; ++b) G[static_cast<size_t>(a) * r + b] += ua * row[b];
    }
  }
  for (int a = 0; a < r; ++a)
    for (int b = 0; b < a; ++b) G[static_cast<size_t>(a) * r + b] = G[static_cast<size_t>(b) * r + a];
  double trace = 0.0;
  for (int a = 0; a < r; ++a) trace += G[static_cast<size_t>(a) * r + a];
  jacobi_eigen(G, V, r);
  std::vector<double> lam(r), scale(r);
  for (int a = 0; a < r; ++a) {
    lam[a] = G[static_cast<size_t>(a) * r + a];
    if (lam[a] > 1e-12 * trace) scale[a] = 1.0 / std::sqrt(lam[a]);
    else { lam[a] = 0.0; scale[a] = 0.0; }                 // rank-deficient direction: no gain there
  }
  const size_t dr = static_cast<size_t>(d) * rpad;
  std::vector<float> h(2 * dr + static_cast<size_t>(T) * rpad + 3 * static_cast<size_t>(T) + rpad + d, 0.f);
  float* hQ = h.data(); float* hQT = hQ + dr; float* hgain = hQT + dr;
  float* hsab = hgain + static_cast<size_t>(T) * rpad; float* hgperp = hsab + T; float* hcoef = hgperp + T;
  float* hqmu = hcoef + T; float* hmu = hqmu + rpad;
  std::vector<double> qmu(r, 0.0), qrow(r);
  for (int i = 0; i < d; ++i) {
    const float* urow = U + static_cast<size_t>(i) * r;
    for (int a = 0; a < r; ++a) qrow[a] = 0.0;
    for (int b = 0; b < r; ++b) {
      const double ub = urow[b];
      const double* vrow = V.data() + static_cast<size_t>(b) * r;
      for (int a = 0; a < r; ++a) qrow[a] += ub * vrow[a];
    }
    for (int a = 0; a < r; ++a) {
      const double q = qrow[a] * scale[a];
      hQ[static_cast<size_t>(i) * rpad + a] = static_cast<float>(q);
      hQT[static_cast<size_t>(a) * d + i] = static_cast<float>(q);
      qmu[a] += q * mu[i];
    }
    hmu[i] = mu[i];
  }
  for (int a = 0; a < r; ++a) hqmu[a] = static_cast<float>(qmu[a]);
  for (int k = 0; k < T; ++k) {
    const double ab = alpha_bar_state[k], sab = std::sqrt(ab), om = 1.0 - ab;
    const double gp = sab * s2 / (ab * s2 + om);
    hsab[k] = static_cast<float>(sab);
    hgperp[k] = static_cast<float>(gp);
    hcoef[k] = static_cast<float>(1.0 - sab * gp);
    for (int a = 0; a < r; ++a) {
      const double ls = lam[a] + s2;
      hgain[static_cast<size_t>(k) * rpad + a] = scale[a] > 0.0 ? static_cast<float>(sab * ls / (ab * ls + om) - gp) : 0.f;
    }
  }
  LowRankDenoiser* L = new (std::nothrow) LowRankDenoiser;
  if (!L) return sdi::fail(E, SD_ERR_ARG, "sdden_lowrank_create: out of host memory");
  L->d = d; L->T = T; L->r = r; L->rpad = rpad;
  {
    // K split of the first product: the largest one (at most 16) that leaves every workgroup 24 slices or more
    const int nk = d / lrgemm::BK;
    for (int ns = 1; ns <= 16; ++ns)
      if (nk % ns == 0 && nk / ns >= 24) L->nsplit = ns;
  }
  hipError_t e = lrgemm::prepare<64, 128, 1, 4, 1, 2>();    // dynamic-LDS limits of the two GEMM stages
  if (e == hipSuccess) e = lrgemm::prepare<64, 128, 1, 4, 2, 2>();
  if (e == hipSuccess) e = hipMalloc(&L->dev, h.size() * sizeof(float));
  if (e == hipSuccess) e = hipMemcpy(L->dev, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    delete L;
    return sdi::fail(E, SD_ERR_HIP, "sdden_lowrank_create: %s", hipGetErrorString(e));
  }
  L->Q = L->dev; L->QT = L->Q + dr; L->gain = L->QT + dr; L->sab = L->gain + static_cast<size_t>(T) * rpad;
  L->gperp = L->sab + T; L->coef = L->gperp + T; L->qmu = L->coef + T; L->mu = L->qmu + rpad;
  *out = L;
  return SD_OK;
}
