// Random-init time-conditioned MLP denoiser: [x ; sinusoidal(k)] -> H -> H -> d, SiLU, bf16 weights
// and activations, fp32 accumulation on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
// All rows of a batched target call (every drafted state of every chain, each at its own step k)
// go through three GEMMs (paper: Alg. "Speculative Sampling for DDM", (Par.) line; Sec. 3.1 for the
// network as a black box).
//
// Data flow per call:
//   compact_rows      rows with krow >= 0 -> dense list (masked drafts cost no MFMA work)
//   gather_convert    X[rowidx[m]] fp32 -> Xb[m] bf16 (dense A operand of layer 1)
//   gemm<1>           H1 = silu(Xb W1x + tb[krow])        tb[k] = b1 + emb(k) W1t, folded at create
//   gemm<2>           H2 = silu(H1 W2 + b2)
//   gemm<3>           out[rowidx[m]] = H2 W3 + b3          (fp32, scattered back to the source rows)
//
// The GEMM kernel (direct global->LDS loads, XOR-swizzled LDS rows, 32x32x16 bf16 MFMA tiles,
// XCD-aware tile order) is in mlp_gemm.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "mlp_gemm.h"
#include "mlp_gemm_pp.h"
#include "sdden_internal.h"
#include "sdden_rows.h"

namespace {

using mlpgemm::to_bf16_bits;
constexpr int kThreads = 256;

// X[rowidx[m], :] fp32 -> Xb[m, :] bf16, 8 elements per thread.
__global__ __launch_bounds__(kThreads) void gather_convert_kernel(const float* __restrict__ X,
                                                                  const int32_t* __restrict__ rowidx,
                                                                  const int32_t* __restrict__ count,
                                                                  uint16_t* __restrict__ Xb, int d) {
  const int M = *count;
  const int per_row = d / 8;
  for (int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
       g < static_cast<int64_t>(M) * per_row; g += static_cast<int64_t>(gridDim.x) * kThreads) {
    const int m = static_cast<int>(g / per_row), c = static_cast<int>(g % per_row);
    const float* src = X + static_cast<int64_t>(rowidx[m]) * d + 8 * c;
    const float4 lo = *reinterpret_cast<const float4*>(src);
    const float4 hi = *reinterpret_cast<const float4*>(src + 4);
    uint4 o;
    o.x = to_bf16_bits(lo.x) | (static_cast<uint32_t>(to_bf16_bits(lo.y)) << 16);
    o.y = to_bf16_bits(lo.z) | (static_cast<uint32_t>(to_bf16_bits(lo.w)) << 16);
    o.z = to_bf16_bits(hi.x) | (static_cast<uint32_t>(to_bf16_bits(hi.y)) << 16);
    o.w = to_bf16_bits(hi.z) | (static_cast<uint32_t>(to_bf16_bits(hi.w)) << 16);
    *reinterpret_cast<uint4*>(Xb + static_cast<int64_t>(m) * d + 8 * c) = o;
  }
}

float bf16_bits_to_float(uint16_t b) {
  const uint32_t u = static_cast<uint32_t>(b) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// Dynamic-LDS limits of every GEMM instantiation launch_gemm can pick, on the current device.
template <int EPI, bool GATHER>
hipError_t prepare_gemms() {
  hipError_t e = mlpgemm::prepare<256, 256, 2, 4, EPI, 2, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare<128, 128, 2, 2, EPI, 2, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare<64, 128, 2, 2, EPI, 2, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare<64, 128, 2, 2, EPI, 4, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare_hs<EPI, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare_pp<EPI, GATHER>();
  if (e == hipSuccess) e = mlpgemm::prepare_pp<EPI, GATHER, 1>();
  if (e == hipSuccess) e = mlpgemm::prepare_pp<EPI, GATHER, 2>();
  if (e == hipSuccess) e = mlpgemm::prepare_pp<EPI, GATHER, 3>();
  if (e == hipSuccess) e = mlpgemm::prepare_pp<EPI, GATHER, 4>();
  return e;
}

// Tile choice by how well the launch fills the 256 CUs.  The 256x256 tile (8 wavefronts, two LDS
// stages) has the highest rate per CU and is taken when its rounds of workgroups are at least 60 % full
// over the whole launch (at 71 % -- 544 tiles in three rounds -- it still runs the call 5 % faster than
// the 128x128 tile does); otherwise 128x128 (4 wavefronts, two stages, two workgroups per CU) when
// that gives 512 tiles or more, else 64x128: with at most one workgroup per CU (the window-start
// call) as a four-stage ring, with more as two stages so that three workgroups share a CU.
template <int EPI, bool GATHER = false>
int launch_gemm(const mlpgemm::Args& a, int R, hipStream_t st, std::string& err, int variant) {
  const int t256 = ((R + 255) / 256) * (a.N / 256);
  const int t128 = ((R + 127) / 128) * (a.N / 128);
  const int t64 = ((R + 63) / 64) * (a.N / 128);
  hipError_t e;
  if (10 * t256 >= 6 * ((t256 + 255) / 256) * 256) {
    if (!mlpgemm::hs_applicable(a)) e = mlpgemm::launch<256, 256, 2, 4, EPI, 2, GATHER>(a, R, st);
    else if (variant == 1) e = mlpgemm::launch_hs<EPI, GATHER>(a, R, st);
    else if (variant == 2) e = mlpgemm::launch_pp<EPI, GATHER, 1>(a, R, st);
    else if (variant == 3) e = mlpgemm::launch_pp<EPI, GATHER, 2>(a, R, st);
    else if (variant == 4) e = mlpgemm::launch_pp<EPI, GATHER, 3>(a, R, st);
    else if (variant == 5) e = mlpgemm::launch_pp<EPI, GATHER, 4>(a, R, st);
    else e = mlpgemm::launch_pp<EPI, GATHER>(a, R, st);
  }
  else if (t128 >= 512) e = mlpgemm::launch<128, 128, 2, 2, EPI, 2, GATHER>(a, R, st);
  else if (t64 > 256) e = mlpgemm::launch<64, 128, 2, 2, EPI, 2, GATHER>(a, R, st);
  else e = mlpgemm::launch<64, 128, 2, 2, EPI, 4, GATHER>(a, R, st);
  if (e != hipSuccess) return sdi::fail(err, SD_ERR_HIP, "mlp gemm launch: %s", hipGetErrorString(e));
  return SD_OK;
}

struct MlpDenoiser final : sdden {
  int H = 0, E = 0;
  uint16_t *W1t = nullptr, *W2t = nullptr, *W3t = nullptr;    // [H,d], [H,H], [d,H] bf16
  float *tb = nullptr, *b2 = nullptr, *b3 = nullptr;          // [T,H], [H], [d]
  int32_t *rowidx = nullptr, *count = nullptr;
  uint16_t *Xb = nullptr, *H1 = nullptr, *H2 = nullptr;
  int cap_rows = 0;
  int gemm_variant = 0;          // 0: kernel_pp; measurement only: 1 = kernel_hs, 2..5 = kernel_pp with pieces left out

  ~MlpDenoiser() override {
    for (void* q : {static_cast<void*>(W1t), static_cast<void*>(W2t), static_cast<void*>(W3t), static_cast<void*>(tb),
                    static_cast<void*>(b2), static_cast<void*>(b3), static_cast<void*>(rowidx), static_cast<void*>(count),
                    static_cast<void*>(Xb), static_cast<void*>(H1), static_cast<void*>(H2)})
      if (q) (void)hipFree(q);
  }

  int reserve(int R) override {
    if (R <= cap_rows) return SD_OK;
    for (void* q : {static_cast<void*>(rowidx), static_cast<void*>(Xb), static_cast<void*>(H1), static_cast<void*>(H2)})
      if (q) (void)hipFree(q);
    rowidx = nullptr; Xb = H1 = H2 = nullptr; cap_rows = 0;
    // the GEMM reads whole tiles of its A operand: round the row capacity up
    const size_t Rp = (static_cast<size_t>(R) + mlpgemm::kRowPad - 1) / mlpgemm::kRowPad * mlpgemm::kRowPad;
    SD_HIP_TRY(err, hipMalloc(&rowidx, sizeof(int32_t) * Rp));
    SD_HIP_TRY(err, hipMalloc(&Xb, 2 * Rp * d));
    SD_HIP_TRY(err, hipMalloc(&H1, 2 * Rp * H));
    SD_HIP_TRY(err, hipMalloc(&H2, 2 * Rp * H));
    SD_HIP_TRY(err, hipMemset(Xb, 0, 2 * Rp * d));
    SD_HIP_TRY(err, hipMemset(H1, 0, 2 * Rp * H));
    SD_HIP_TRY(err, hipMemset(H2, 0, 2 * Rp * H));
    if (!count) SD_HIP_TRY(err, hipMalloc(&count, sizeof(int32_t)));
    cap_rows = R;
    return SD_OK;
  }

  int eval(int R, const float* X, const int32_t* krow, float* out, hipStream_t st) override {
    return eval_impl(R, X, nullptr, krow, out, st);
  }
  int eval_mirror(int R, const float* X, const uint16_t* Xbf16, const int32_t* krow, float* out, hipStream_t st) override {
    return eval_impl(R, X, Xbf16, krow, out, st);
  }

  // With a bf16 image of the rows the first GEMM gathers its A rows from it and no conversion pass runs.
  int eval_impl(int R, const float* X, const uint16_t* Xbf16, const int32_t* krow, float* out, hipStream_t st) {
    if (R > cap_rows)
      return sdi::fail(err, SD_ERR_WORKSPACE, "sdden_eval(mlp): %d rows exceed the %d reserved (sdden_reserve)", R, cap_rows);
    if (!sdi::aligned16(X) || !sdi::aligned16(out))
      return sdi::fail(err, SD_ERR_ARG, "sdden_eval(mlp): X and out must be 16-byte aligned");
    if (Xbf16 && !sdi::aligned16(Xbf16))
      return sdi::fail(err, SD_ERR_ARG, "sdden_eval_mirror(mlp): Xbf16 must be 16-byte aligned");
    hipLaunchKernelGGL(sdrows::compact_rows_kernel, dim3(sdrows::compact_rows_grid(R)), dim3(sdrows::kScan), 0, st, krow, rowidx, count,
                       active, rows_per_chain, R, T);
    mlpgemm::Args a;
    a.count = count; a.rowidx = rowidx; a.krow = krow; a.arow = nullptr;
    int rc;
    a.Bt = W1t; a.N = H; a.Kdim = d; a.bias = tb; a.outb = H1; a.outf = nullptr;
    if (Xbf16) {
      a.A = Xbf16; a.arow = rowidx;
      prof.mark(1, st);
      rc = launch_gemm<1, true>(a, R, st, err, gemm_variant);
      prof.mark(1, st);
    } else {
      const int64_t chunks = static_cast<int64_t>(R) * (d / 8);
      const int cgrid = static_cast<int>(std::min<int64_t>((chunks + kThreads - 1) / kThreads, 256 * 32));
      hipLaunchKernelGGL(gather_convert_kernel, dim3(cgrid), dim3(kThreads), 0, st, X, rowidx, count, Xb, d);
      a.A = Xb;
      prof.mark(1, st);
      rc = launch_gemm<1>(a, R, st, err, gemm_variant);
      prof.mark(1, st);
    }
    a.arow = nullptr;
    if (rc) return rc;
    a.A = H1; a.Bt = W2t; a.N = H; a.Kdim = H; a.bias = b2; a.outb = H2;
    prof.mark(2, st);
    rc = launch_gemm<2>(a, R, st, err, gemm_variant);
    prof.mark(2, st);
    if (rc) return rc;
    a.A = H2; a.Bt = W3t; a.N = d; a.Kdim = H; a.bias = b3; a.outb = nullptr; a.outf = out;
    prof.mark(3, st);
    rc = launch_gemm<3>(a, R, st, err, gemm_variant);
    prof.mark(3, st);
    if (rc) return rc;
    SD_HIP_TRY(err, hipGetLastError());
    return SD_OK;
  }
};

// dst[n][k] = src[k][n] for a [K, N] bf16 matrix.
void transpose_bits(const uint16_t* src, int K, int N, std::vector<uint16_t>& dst) {
  dst.resize(static_cast<size_t>(K) * N);
  constexpr int TB = 64;
  for (int k0 = 0; k0 < K; k0 += TB)
    for (int n0 = 0; n0 < N; n0 += TB)
      for (int k = k0; k < std::min(K, k0 + TB); ++k)
        for (int n = n0; n < std::min(N, n0 + TB); ++n)
          dst[static_cast<size_t>(n) * K + k] = src[static_cast<size_t>(k) * N + n];
}

}  // namespace

extern "C" int sdden_mlp_create(int32_t d, int32_t H, int32_t E, const uint16_t* W1, const float* b1,
                                const uint16_t* W2, const float* b2, const uint16_t* W3, const float* b3,
                                int32_t T, int32_t Rmax, sdden** out) {
  std::string& ER = sdi::g_den_create_error;
  if (!W1 || !b1 || !W2 || !b2 || !W3 || !b3 || !out || d <= 0 || H <= 0 || E < 0 || (E & 1) || T <= 0 || Rmax <= 0)
    return sdi::fail(ER, SD_ERR_ARG, "sdden_mlp_create: bad argument");
  if (d % 256 != 0 || H % 256 != 0)
    return sdi::fail(ER, SD_ERR_UNSUPPORTED, "sdden_mlp_create: d=%d and H=%d must be multiples of 256", d, H);
  MlpDenoiser* m = new (std::nothrow) MlpDenoiser;
  if (!m) return sdi::fail(ER, SD_ERR_ARG, "sdden_mlp_create: out of host memory");
  m->d = d; m->T = T; m->H = H; m->E = E;
  // per-step bias table: tb[k] = b1 + emb(k) . W1[d:d+E, :],  emb = [sin(k w_i) ; cos(k w_i)], w_i = 10000^(-2i/E)
  std::vector<float> tb(static_cast<size_t>(T) * H);
  {
    const int half = E / 2;
    std::vector<double> emb(E > 0 ? E : 1), row(H);
    for (int k = 0; k < T; ++k) {
      for (int i = 0; i < half; ++i) {
        const double w = std::pow(10000.0, -static_cast<double>(i) / half);
        emb[i] = std::sin(k * w);
        emb[half + i] = std::cos(k * w);
      }
      for (int n = 0; n < H; ++n) row[n] = b1[n];
      for (int e = 0; e < E; ++e) {
        const uint16_t* wrow = W1 + static_cast<size_t>(d + e) * H;
        const double ev = emb[e];
        for (int n = 0; n < H; ++n) row[n] += ev * bf16_bits_to_float(wrow[n]);
      }
      for (int n = 0; n < H; ++n) tb[static_cast<size_t>(k) * H + n] = static_cast<float>(row[n]);
    }
  }
  std::vector<uint16_t> w1t, w2t, w3t;
  transpose_bits(W1, d, H, w1t);      // first d rows of W1 only: [d,H] -> [H,d]
  transpose_bits(W2, H, H, w2t);
  transpose_bits(W3, H, d, w3t);      // [H,d] -> [d,H]
  hipError_t e = prepare_gemms<1, false>();
  if (e == hipSuccess) e = prepare_gemms<1, true>();
  if (e == hipSuccess) e = prepare_gemms<2, false>();
  if (e == hipSuccess) e = prepare_gemms<3, false>();
  auto up = [&](auto** dst, const void* src, size_t bytes) {
    if (e != hipSuccess) return;
    e = hipMalloc(reinterpret_cast<void**>(dst), bytes);
    if (e == hipSuccess) e = hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice);
  };
  up(&m->W1t, w1t.data(), w1t.size() * 2);
  up(&m->W2t, w2t.data(), w2t.size() * 2);
  up(&m->W3t, w3t.data(), w3t.size() * 2);
  up(&m->tb, tb.data(), tb.size() * 4);
  up(&m->b2, b2, static_cast<size_t>(H) * 4);
  up(&m->b3, b3, static_cast<size_t>(d) * 4);
  if (e != hipSuccess) {
    delete m;
    return sdi::fail(ER, SD_ERR_HIP, "sdden_mlp_create: %s", hipGetErrorString(e));
  }
  if (int rc = m->reserve(Rmax)) {
    ER = m->err;
    delete m;
    return rc;
  }
  *out = m;
  return SD_OK;
}

// Measurement aid: which kernel serves the 256 x 256 tile (0 = default, 1 = kernel_hs).
extern "C" int sdden_mlp_select_gemm(sdden* den, int32_t variant) {
  MlpDenoiser* m = dynamic_cast<MlpDenoiser*>(den);
  if (!m) return SD_ERR_ARG;
  if (variant < 0 || variant > 5) return sdi::fail(m->err, SD_ERR_ARG, "sdden_mlp_select_gemm: variant must be 0..5");
  m->gemm_variant = variant;
  return SD_OK;
}
