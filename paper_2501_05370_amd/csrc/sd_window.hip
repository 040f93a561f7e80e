// Window kernels of speculative sampling for diffusion chains (gfx950) and their C entry points:
// initial state, frozen draft rollout, accept / first-reject / reflect, advance + compaction.
//
// Paper: Alg. "Speculative Sampling for DDM", Alg. "REJECTION ... two Gaussians with same
// covariance" (reflection maximal coupling), and the detailed algorithm of the appendix.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>
#include <new>

#include "sd_internal.h"
#include "sd_lanes.h"
#include "sd_rng.h"

namespace {

constexpr int kBlock = 256;   // threads per workgroup (4 wavefronts of 64)

std::string g_create_error;

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------
template <int VEC>
struct Pack;
template <>
struct Pack<4> {
  float v[4];
  __device__ __forceinline__ void load(const float* p) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ __forceinline__ void store(float* p) const {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct Pack<1> {
  float v[1];
  __device__ __forceinline__ void load(const float* p) { v[0] = *p; }
  __device__ __forceinline__ void store(float* p) const { *p = v[0]; }
};

__device__ __forceinline__ int active_chains(const int32_t* active, int B) {
  if (active == nullptr) return B;
  const int a = *active;
  return a < B ? (a < 0 ? 0 : a) : B;
}

// Sum over the `WIDTH` consecutive lanes this lane belongs to; every lane gets the total.
template <int WIDTH>
__device__ __forceinline__ double group_sum(double v) {
  if constexpr (WIDTH >= 2) v += sdlane::lane_xor<1>(v);
  if constexpr (WIDTH >= 4) v += sdlane::lane_xor<2>(v);
  if constexpr (WIDTH >= 8) v += sdlane::lane_xor<4>(v);
  if constexpr (WIDTH >= 16) v += sdlane::lane_xor<8>(v);
  if constexpr (WIDTH >= 32) v = sdlane::pair_sum_rows<16>(v);
  if constexpr (WIDTH >= 64) v = sdlane::pair_sum_rows<32>(v);
  return v;
}

// ---------------------------------------------------------------------------------------------
// Y_0 ~ N(0, Id)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void init_state_kernel(const int64_t* __restrict__ chain_id,
                                                            float* __restrict__ y,
                                                            int32_t* __restrict__ n, int B, int d,
                                                            int nblk, uint64_t seed) {
  const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  if (g >= static_cast<int64_t>(B) * nblk) return;
  const int b = static_cast<int>(g / nblk);
  const int blk = static_cast<int>(g % nblk);
  float z[4];
  sdrng::normal4(seed, chain_id[b], 0u, sdrng::kStreamInit, static_cast<uint32_t>(blk), z);
  float* row = y + static_cast<int64_t>(b) * d;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (4 * blk + e < d) row[4 * blk + e] = z[e];
  if (blk == 0) n[b] = 0;
}

// ---------------------------------------------------------------------------------------------
// Frozen draft rollout: one thread owns one Philox block (4 elements) of one chain and walks
// the window, so the recurrence stays in registers and every drafted element is written once.
// ---------------------------------------------------------------------------------------------
struct DraftArgs {
  const float *y, *D0;
  const int32_t* n;
  const int64_t* id;
  float* Ytil;
  uint16_t* mirror;      // optional bf16 image of Ytil (round-to-nearest-even), same layout
  int32_t* krow;
  const float *a, *c, *sigma;
  const int32_t* active;
  int B, d, K, T, nblk;
  int rs, roff;          // window rows per chain in Ytil / krow and the row the first draft goes to
                         // (K, 0; or K+1, 1 with row 0 = a copy of y for the one batched target call)
  uint64_t seed;
};

__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
  const __bf16 a = static_cast<__bf16>(lo), b = static_cast<__bf16>(hi);
  uint16_t ua, ub;
  __builtin_memcpy(&ua, &a, 2);
  __builtin_memcpy(&ub, &b, 2);
  return static_cast<uint32_t>(ua) | (static_cast<uint32_t>(ub) << 16);
}

template <int VEC>
__device__ __forceinline__ void store_mirror(uint16_t* dst, const float v[4], int i0, int d) {
  if (VEC == 4) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(bf16_pair(v[0], v[1]), bf16_pair(v[2], v[3]));
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (i0 + e < d) dst[e] = static_cast<uint16_t>(bf16_pair(v[e], 0.f) & 0xffffu);
  }
}

template <int VEC>
__global__ __launch_bounds__(kBlock) void draft_frozen_kernel(DraftArgs p) {
  const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  const int Bact = active_chains(p.active, p.B);
  if (g >= static_cast<int64_t>(Bact) * p.nblk) return;
  const int b = static_cast<int>(g / p.nblk);
  const int blk = static_cast<int>(g % p.nblk);
  const int i0 = 4 * blk;
  const int n = p.n[b];
  const int Kt = min(p.K, p.T - n);
  const int64_t id = p.id[b];

  float prev[4], d0[4];
  const int64_t row0 = static_cast<int64_t>(b) * p.d + i0;
  if (VEC == 4) {
    Pack<4> t;
    t.load(p.y + row0);
#pragma unroll
    for (int e = 0; e < 4; ++e) prev[e] = t.v[e];
    t.load(p.D0 + row0);
#pragma unroll
    for (int e = 0; e < 4; ++e) d0[e] = t.v[e];
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool in = i0 + e < p.d;
      prev[e] = in ? p.y[row0 + e] : 0.f;
      d0[e] = in ? p.D0[row0 + e] : 0.f;
    }
  }
  if (p.roff) {                         // row 0 of the chain's block: the window-start state itself
    float* dst = p.Ytil + static_cast<int64_t>(b) * p.rs * p.d + i0;
    if (VEC == 4) {
      *reinterpret_cast<float4*>(dst) = make_float4(prev[0], prev[1], prev[2], prev[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (i0 + e < p.d) dst[e] = prev[e];
    }
    if (p.mirror) store_mirror<VEC>(p.mirror + static_cast<int64_t>(b) * p.rs * p.d + i0, prev, i0, p.d);
    if (blk == 0) p.krow[static_cast<int64_t>(b) * p.rs] = n < p.T ? n : -1;   // a finished chain asks for no prediction
  }
  for (int j = 0; j < p.K; ++j) {       // position j+1 of the window, produces state n+j+1
    float out[4] = {0.f, 0.f, 0.f, 0.f};
    if (j < Kt) {
      const int k = n + j;
      const float a = p.a[k], c = p.c[k], s = p.sigma[k];
      float z[4];
      sdrng::normal4(p.seed, id, static_cast<uint32_t>(k + 1), sdrng::kStreamNoise,
                     static_cast<uint32_t>(blk), z);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        prev[e] = fmaf(a, prev[e], fmaf(c, d0[e], s * z[e]));
        out[e] = prev[e];
      }
    }
    float* dst = p.Ytil + (static_cast<int64_t>(b) * p.rs + p.roff + j) * p.d + i0;
    if (VEC == 4) {
      *reinterpret_cast<float4*>(dst) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (i0 + e < p.d) dst[e] = out[e];
    }
    if (p.mirror) store_mirror<VEC>(p.mirror + (static_cast<int64_t>(b) * p.rs + p.roff + j) * p.d + i0, out, i0, p.d);
    if (blk == 0) {
      // which drafted states the target must evaluate: all but the last one; with the extra row also the
      // last one (its prediction is the next window's frozen vector) unless it is the chain's final state
      const bool need = p.roff ? (j + 1 <= Kt && n + j + 1 < p.T) : (j + 1 <= Kt - 1);
      p.krow[static_cast<int64_t>(b) * p.rs + p.roff + j] = need ? n + j + 1 : -1;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One position of a drafter that needs a network call per position (the independent draft model
// of Sec. 3.1): m^p = a_k prev + c_k D^p(prev, k), y~ = m^p + sigma_k z_{k+1}, k = n + j - 1.
// Same thread-per-Philox-block mapping and noise keys as the frozen rollout.  Besides the window
// rows it writes the new state as a dense [B,d] matrix and its step index, the input of the
// drafter's next call (index -1 once the chain's window has ended).
// ---------------------------------------------------------------------------------------------
struct DraftStepArgs {
  const float *prev, *Dp;
  const int32_t* n;
  const int64_t* id;
  float *mp, *Ytil, *next;
  int32_t *krow, *knext;
  const float *a, *c, *sigma;
  const int32_t* active;
  int B, d, K, T, nblk, j;
  uint64_t seed;
};

template <int VEC>
__global__ __launch_bounds__(kBlock) void draft_step_kernel(DraftStepArgs p) {
  const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
  const int Bact = active_chains(p.active, p.B);
  if (g >= static_cast<int64_t>(Bact) * p.nblk) return;
  const int b = static_cast<int>(g / p.nblk);
  const int blk = static_cast<int>(g % p.nblk);
  const int i0 = 4 * blk;
  const int n = p.n[b];
  const int Kt = min(p.K, p.T - n);
  const int j = p.j;                                  // 1-based window position
  float m[4] = {0.f, 0.f, 0.f, 0.f}, out[4] = {0.f, 0.f, 0.f, 0.f};
  const int64_t row = static_cast<int64_t>(b) * p.d + i0;
  if (j <= Kt) {
    const int k = n + j - 1;
    const float a = p.a[k], c = p.c[k], s = p.sigma[k];
    float pv[4], dp[4], z[4];
    if (VEC == 4) {
      Pack<4> t;
      t.load(p.prev + row);
#pragma unroll
      for (int e = 0; e < 4; ++e) pv[e] = t.v[e];
      t.load(p.Dp + row);
#pragma unroll
      for (int e = 0; e < 4; ++e) dp[e] = t.v[e];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = i0 + e < p.d;
        pv[e] = in ? p.prev[row + e] : 0.f;
        dp[e] = in ? p.Dp[row + e] : 0.f;
      }
    }
    sdrng::normal4(p.seed, p.id[b], static_cast<uint32_t>(k + 1), sdrng::kStreamNoise, static_cast<uint32_t>(blk), z);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      m[e] = fmaf(a, pv[e], c * dp[e]);
      out[e] = fmaf(s, z[e], m[e]);
    }
  }
  const int64_t w = (static_cast<int64_t>(b) * p.K + (j - 1)) * p.d + i0;
  if (VEC == 4) {
    *reinterpret_cast<float4*>(p.mp + w) = make_float4(m[0], m[1], m[2], m[3]);
    *reinterpret_cast<float4*>(p.Ytil + w) = make_float4(out[0], out[1], out[2], out[3]);
    if (p.next) *reinterpret_cast<float4*>(p.next + row) = make_float4(out[0], out[1], out[2], out[3]);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (i0 + e < p.d) {
        p.mp[w + e] = m[e];
        p.Ytil[w + e] = out[e];
        if (p.next) p.next[row + e] = out[e];
      }
  }
  if (blk == 0) {
    const int kn = (j <= Kt - 1) ? n + j : -1;
    p.krow[static_cast<int64_t>(b) * p.K + (j - 1)] = kn;
    if (p.knext) p.knext[b] = kn;
  }
}

// ---------------------------------------------------------------------------------------------
// Accept test, first rejection, reflection.
//
// TPC threads cooperate on one chain (one chain per workgroup from 256 threads up, several below).  Pass 1
// streams the chain's rows of drafts and target predictions: a thread owns a set of 16-byte columns and walks
// the window positions JC at a time, keeping the previous row in registers, and accumulates the two dot products
// of every position in fp64.  The per-position sums are reduced with wavefront exchanges (and LDS across
// wavefronts), the first JC lanes of the chain run the accept test of one position each, and a ballot finds the
// first rejection; the groups of JC positions after it are not read (unless the per-position diagnostics are
// asked for).  Pass 2 re-reads only the rejected row and writes the reflected state (or copies the last draft).
//
// What bounds the kernel once the first groups of all chains have streamed is the chain with the latest
// rejection: its groups are dependent steps (load, reduce, decide).  Hence the loads of UNR columns are requested
// together before any arithmetic, the logs of the window's accept-test uniforms are drawn once up front by one
// lane per position, off the steps' critical path, and 512 threads share a chain at d = 12288 (two workgroups
// per CU keep all 512 chains resident; 1024 threads per chain leave one workgroup per CU, whose load and reduce
// phases then have nothing to overlap with, and measured slower).
//
// Loop bounds depend on K and on per-workgroup flags only, so every barrier and shuffle is reached by all threads.
// ---------------------------------------------------------------------------------------------
struct VerifyArgs {
  const float *y, *D0mp, *Dq, *Ytil;
  int rs, roff;                // rows per chain of Ytil / Dq, row of the first draft in Ytil (see DraftArgs)
  int first_exact;             // FROZEN: D0 is the target's prediction at y, so Delta_1 = 0 and row 0 of Dq is not read
  const float* Dq0;            // EXPLICIT mode, optional: row 0 of Dq kept as a separate [B,d] array
  const int32_t* n;
  const int64_t* id;
  float* y_out;
  int32_t* adv;
  uint8_t* rej;
  float *logratio, *logu;
  const float *a, *c, *sigma;
  const int32_t* active;
  int B, d, K, T;
  uint64_t seed;
  double inv_tau;
};

// Shared state of one chain's threads during pass 1.
template <int CPW, int WMAX>
struct VerifyShared {
  double part[WMAX][16];                 // per-wavefront partial sums of a group (2 * JC <= 16)
  int jr[CPW];                           // first rejected position so far, -1 = none
  double coef[CPW];                      // Z.Delta / |Delta|^2 at that position
  double lu[CPW][SD_MAX_WINDOW];         // log u of every window position
};

// Per-chain constants of pass 1.
struct VerifyChain {
  int b, n, Kt, ncol, slot, t;
  bool valid, skip0, need_all;
  int64_t rowB, winB, yoff;
};

// Positions jc .. jc+JC-1 of one chain: stream their rows (UNR columns per thread requested together), reduce
// the two dot products of every position, run the accept tests and record the first rejection.  Every thread
// of the workgroup calls this with the same jc (it holds workgroup barriers).
template <int TPC, int VEC, bool FROZEN, int JC, int UNR, typename Shared>
__device__ __forceinline__ void verify_group(const VerifyArgs& p, const VerifyChain& c, Shared& sh, int jc) {
  constexpr int WAVES = TPC / 64;
  constexpr int WIDTH = TPC < 64 ? TPC : 64;
  constexpr int MU = FROZEN ? 1 : UNR, MJ = FROZEN ? 1 : JC;   // the explicit draft means are loaded like the drafts
  static_assert(TPC >= JC && 2 * JC <= 16, "one lane per window position of a group");
  const int t = c.t, n = c.n, Kt = c.Kt, slot = c.slot;
  float ak[JC], ck[JC];
#pragma unroll
  for (int jj = 0; jj < JC; ++jj) {
    const bool in = jc + jj < Kt;
    ak[jj] = in ? p.a[n + jc + jj] : 0.f;
    ck[jj] = in ? p.c[n + jc + jj] : 0.f;
  }
  double s1[JC], s2[JC];
#pragma unroll
  for (int jj = 0; jj < JC; ++jj) s1[jj] = s2[jj] = 0.0;

  // a group after the chain's first rejection decides nothing: it is streamed only when the caller asked
  // for the per-position log-ratios (jr was last written before the barrier that ended the previous group)
  if (jc < Kt && (c.need_all || sh.jr[slot] < 0)) {
    const float* prow = jc == 0 ? p.y + c.rowB : p.Ytil + c.winB + c.yoff + static_cast<int64_t>(jc - 1) * p.d;
    for (int col0 = t; col0 < c.ncol; col0 += TPC * UNR) {
      Pack<VEC> prev[UNR], d0[UNR], cur[UNR][JC], dq[UNR][JC], mp[MU][MJ];
      // every load of the UNR columns is requested before the first product
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int col = col0 + u * TPC;
        if (UNR > 1 && col >= c.ncol) continue;
        const int64_t off = static_cast<int64_t>(col) * VEC;
        prev[u].load(prow + off);
        if (FROZEN) d0[u].load(p.D0mp + c.rowB + off);
#pragma unroll
        for (int jj = 0; jj < JC; ++jj) {
          const int j = jc + jj;
          if (j < Kt) {
            const int64_t r = c.winB + static_cast<int64_t>(j) * p.d + off;
            cur[u][jj].load(p.Ytil + r + c.yoff);
            if (FROZEN) {
              if (j > 0 || !c.skip0) dq[u][jj].load(p.Dq + r);
            } else {
              if (j == 0 && p.Dq0) dq[u][jj].load(p.Dq0 + c.rowB + off);
              else dq[u][jj].load(p.Dq + r);
              mp[FROZEN ? 0 : u][FROZEN ? 0 : jj].load(p.D0mp + r);
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int col = col0 + u * TPC;
        if (UNR > 1 && col >= c.ncol) continue;
#pragma unroll
        for (int jj = 0; jj < JC; ++jj) {
          const int j = jc + jj;
          if (j < Kt) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              double w, dl;      // w = sigma*Z, dl = (sigma/c)*Delta (FROZEN) or sigma*Delta
              const float pv = jj == 0 ? prev[u].v[e] : cur[u][jj > 0 ? jj - 1 : 0].v[e];
              if (FROZEN) {
                w = static_cast<double>(cur[u][jj].v[e]) - static_cast<double>(ak[jj]) * pv -
                    static_cast<double>(ck[jj]) * d0[u].v[e];
                dl = (j > 0 || !c.skip0) ? static_cast<double>(d0[u].v[e]) - static_cast<double>(dq[u][jj].v[e]) : 0.0;
              } else {
                const float m = mp[FROZEN ? 0 : u][FROZEN ? 0 : jj].v[e];
                w = static_cast<double>(cur[u][jj].v[e]) - static_cast<double>(m);
                dl = static_cast<double>(m) - (static_cast<double>(ak[jj]) * pv +
                                               static_cast<double>(ck[jj]) * dq[u][jj].v[e]);
              }
              s1[jj] = fma(w, dl, s1[jj]);
              s2[jj] = fma(dl, dl, s2[jj]);
            }
          }
        }
      }
    }
  }

  // ---- reduce the 2*JC sums over the chain's threads
  double mine1 = 0.0, mine2 = 0.0;      // lane t < JC ends up with the sums of position jc+t
#pragma unroll
  for (int jj = 0; jj < JC; ++jj) {
    s1[jj] = group_sum<WIDTH>(s1[jj]);
    s2[jj] = group_sum<WIDTH>(s2[jj]);
  }
  if (WAVES > 1) {
    const int wave = t / 64;
    if ((t & 63) == 0) {
#pragma unroll
      for (int jj = 0; jj < JC; ++jj) {
        sh.part[wave][jj] = s1[jj];
        sh.part[wave][JC + jj] = s2[jj];
      }
    }
    __syncthreads();
    if (t < JC) {
#pragma unroll
      for (int w = 0; w < (WAVES > 1 ? WAVES : 1); ++w) {
        mine1 += sh.part[w][t];
        mine2 += sh.part[w][JC + t];
      }
    }
  } else {
#pragma unroll
    for (int jj = 0; jj < JC; ++jj)
      if (t == jj) { mine1 = s1[jj]; mine2 = s2[jj]; }
  }

  // ---- accept test of position j = jc + t by the chain's first JC lanes
  bool reject = false;
  double coef = 0.0;
  if (t < JC) {
    const int j = jc + t;
    const bool inwin = j < Kt;
    double lr = 0.0, lu = 0.0;
    if (inwin) {
      const int k = n + j;
      const double sg = p.sigma[k];
      const double inv_s2 = 1.0 / (sg * sg);
      double S1, S2;                       // Z.Delta and |Delta|^2
      if (FROZEN) {
        const double cc = p.c[k];
        S1 = mine1 * cc * inv_s2;
        S2 = mine2 * cc * cc * inv_s2;
      } else {
        S1 = mine1 * inv_s2;
        S2 = mine2 * inv_s2;
      }
      lr = (-S1 - 0.5 * S2) * p.inv_tau;
      lu = sh.lu[slot][j];
      // a log-ratio that is not a number (non-finite inputs) counts as a rejection
      reject = !(S2 == 0.0 || (lr == lr && lu <= fmin(0.0, lr)));
      coef = S2 > 0.0 ? S1 / S2 : 0.0;
    }
    if (c.valid && j < p.K) {
      if (p.logratio) p.logratio[static_cast<int64_t>(c.b) * p.K + j] = static_cast<float>(lr);
      if (p.logu) p.logu[static_cast<int64_t>(c.b) * p.K + j] = static_cast<float>(lu);
    }
  }
  const unsigned long long ballot = __ballot(reject);
  const int lane = threadIdx.x & 63;
  const unsigned long long mine =
      (TPC < 64) ? ((ballot >> (lane & ~(TPC - 1))) & ((1ull << JC) - 1ull)) : (ballot & ((1ull << JC) - 1ull));
  if (t < JC && reject && sh.jr[slot] < 0 && (mine & ((1ull << t) - 1ull)) == 0ull) {
    // lowest rejecting position of this group, and no earlier group rejected
    sh.jr[slot] = jc + t;
    sh.coef[slot] = coef;
  }
  __syncthreads();
}

// GROUPS: 0 = groups of 4 positions, one column at a time (short rows; the explicit-mean form, which carries one
// more operand row per position); 1 = groups of 2 positions, 3 columns at a time (the same number of loads
// outstanding per thread): most chains reject within the first positions, where a small group reads fewer rows
// past the rejection.  A thread adds its columns in the same order whatever the grouping, so the schedules give
// bit-identical sums.  Measured and dropped: groups growing 2, 2, 4, 8 (the widest group sets the register count,
// 157 against 108, and the lost occupancy costs more than the steps save) and 2, 2, then 4 (in the c4 sampler 79.5
// against 77.3 us per launch: a group of 4 goes one column at a time, and the steps of a long chain are bound by
// the loads one workgroup keeps in flight, not by their number).
template <int TPC, int VEC, bool FROZEN, int GROUPS>
__global__ __launch_bounds__(TPC > kBlock ? TPC : kBlock) void verify_kernel(VerifyArgs p) {
  constexpr int BLOCK = TPC > kBlock ? TPC : kBlock;
  constexpr int CPW = BLOCK / TPC;                  // chains per workgroup
  constexpr int WAVES = TPC / 64;                   // wavefronts per chain (0: sub-wavefront)
  __shared__ VerifyShared<CPW, (WAVES > 1 ? WAVES : 1)> sh;

  VerifyChain c;
  c.slot = TPC == BLOCK ? 0 : threadIdx.x / TPC;    // whole workgroup on one chain: uniform
  c.t = threadIdx.x % TPC;
  const int b_raw = blockIdx.x * CPW + c.slot;
  const int Bact = active_chains(p.active, p.B);
  c.valid = b_raw < Bact;
  c.b = c.valid ? b_raw : 0;
  c.n = c.valid ? p.n[c.b] : 0;
  c.Kt = c.valid ? max(0, min(p.K, p.T - c.n)) : 0;
  const int64_t id = c.valid ? p.id[c.b] : 0;
  c.ncol = p.d / VEC;
  c.rowB = static_cast<int64_t>(c.b) * p.d;                  // offset of y[b], D0[b]
  c.winB = static_cast<int64_t>(c.b) * p.rs * p.d;           // offset of the chain's rows in Ytil, Dq
  c.yoff = static_cast<int64_t>(p.roff) * p.d;               // first draft within the chain's rows of Ytil
  c.skip0 = FROZEN && p.first_exact;
  c.need_all = p.logratio != nullptr || p.logu != nullptr;
  const int t = c.t, slot = c.slot, n = c.n, Kt = c.Kt, b = c.b, ncol = c.ncol;
  const bool valid = c.valid;
  const int64_t rowB = c.rowB, winB = c.winB, yoff = c.yoff;

  if (t == 0) sh.jr[slot] = -1;
  for (int j = t; j < Kt; j += TPC)
    sh.lu[slot][j] = sdrng::log_uniform(p.seed, id, static_cast<uint32_t>(n + j + 1));
  __syncthreads();

  // With the whole workgroup on one chain the walk ends at the chain's first rejection (uniform: every thread
  // reads the same flag behind the group's closing barrier) unless the diagnostics want every position; where
  // several chains share a workgroup the later groups only cost their barriers.
  constexpr bool kLeave = TPC == BLOCK;
  if constexpr (GROUPS == 0) {
    for (int jc = 0; jc < p.K; jc += 4) {
      verify_group<TPC, VEC, FROZEN, 4, 1>(p, c, sh, jc);
      if (kLeave && !c.need_all && sh.jr[slot] >= 0) break;
    }
  } else {
    for (int jc = 0; jc < p.K; jc += 2) {
      verify_group<TPC, VEC, FROZEN, 2, 3>(p, c, sh, jc);
      if (kLeave && !c.need_all && sh.jr[slot] >= 0) break;
    }
  }

  // ---- pass 2: write the state the chain keeps
  const int jr = sh.jr[slot];
  if (!valid) return;
  if (t == 0) {
    p.adv[b] = jr >= 0 ? jr + 1 : Kt;
    if (p.rej) p.rej[b] = jr >= 0 ? 1 : 0;
  }
  float* dst = p.y_out + rowB;
  if (jr < 0) {
    const float* src = Kt > 0 ? p.Ytil + winB + yoff + static_cast<int64_t>(Kt - 1) * p.d : p.y + rowB;
    for (int col = t; col < ncol; col += TPC) {
      Pack<VEC> v;
      v.load(src + static_cast<int64_t>(col) * VEC);
      v.store(dst + static_cast<int64_t>(col) * VEC);
    }
    return;
  }
  const int k = n + jr;
  const double a = p.a[k], cc = p.c[k];
  const double two_coef = 2.0 * sh.coef[slot];
  const int64_t r = winB + static_cast<int64_t>(jr) * p.d;
  if (FROZEN) {
    // Y = m^q + sigma (Z - 2 (Z.Delta/|Delta|^2) Delta) with sigma Z = y~ - m^p and sigma Delta = m^p - m^q =
    // c (D0 - Dq): the a * (previous state) terms cancel, Y = y~ - c (1 + 2 Z.Delta/|Delta|^2) (D0 - Dq)
    const double f = cc * (1.0 + two_coef);
    for (int col = t; col < ncol; col += TPC) {
      const int64_t off = static_cast<int64_t>(col) * VEC;
      Pack<VEC> cur, dq, x, o;
      cur.load(p.Ytil + r + yoff + off);
      dq.load(p.Dq + r + off);
      x.load(p.D0mp + rowB + off);
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        o.v[e] = static_cast<float>(static_cast<double>(cur.v[e]) -
                                    f * (static_cast<double>(x.v[e]) - static_cast<double>(dq.v[e])));
      o.store(dst + off);
    }
    return;
  }
  const float* prevrow = jr == 0 ? p.y + rowB : p.Ytil + winB + yoff + static_cast<int64_t>(jr - 1) * p.d;
  for (int col = t; col < ncol; col += TPC) {
    const int64_t off = static_cast<int64_t>(col) * VEC;
    Pack<VEC> prev, cur, dq, x, o;
    prev.load(prevrow + off);
    cur.load(p.Ytil + r + yoff + off);
    if (jr == 0 && p.Dq0) dq.load(p.Dq0 + rowB + off);
    else dq.load(p.Dq + r + off);
    x.load(p.D0mp + r + off);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const double mq = a * prev.v[e] + cc * dq.v[e];
      const double mp = static_cast<double>(x.v[e]);
      // Y = m^q + sigma (Z - 2 (Z.Delta/|Delta|^2) Delta),  sigma Z = cur - m^p, sigma Delta = m^p - m^q
      o.v[e] = static_cast<float>(mq + (static_cast<double>(cur.v[e]) - mp) - two_coef * (mp - mq));
    }
    o.store(dst + off);
  }
}

// ---------------------------------------------------------------------------------------------
// Advance + compaction, in two launches with no wait between workgroups.
// advance_rank_kernel: one workgroup per 1024 chains.  A chain that goes on gets its rank among the
// survivors of its own workgroup (wavefront ballots + a prefix over the 16 wavefront totals); every
// chain's new step and id are parked in the workspace (so that n and chain_id can be rewritten in place
// afterwards), the workgroup's survivor count goes to totals[workgroup], the statistics to the counters.
// advance_move_kernel: a chain's destination is the sum of the totals of the workgroups before its own
// plus its rank (a stable compaction to the front); it moves the state row (and the carried prediction)
// and rewrites n and chain_id.  Rows between the device-side chain count and B get rank -2 and are
// skipped; workgroup 0 writes the new chain count.
// ---------------------------------------------------------------------------------------------
constexpr int kScanBlock = 1024;
constexpr int kScanWaves = kScanBlock / 64;

__global__ __launch_bounds__(kScanBlock) void advance_rank_kernel(
    const int32_t* __restrict__ adv, const uint8_t* __restrict__ rej, const int32_t* __restrict__ n,
    const int64_t* __restrict__ chain_id, int32_t* __restrict__ rank, int32_t* __restrict__ n_new,
    int64_t* __restrict__ id_all, int32_t* __restrict__ totals, int64_t* counters, const int32_t* active, int B,
    int T, int K) {
  __shared__ int wave_tot[kScanWaves];
  __shared__ long long sh_cnt[3];
  const int Bact = active_chains(active, B);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x * kScanBlock + tid;
  if (tid == 0) sh_cnt[0] = sh_cnt[1] = sh_cnt[2] = 0;
  const bool in = b < Bact;
  int nn = 0;
  long long my_adv = 0, my_rej = 0, my_kt = 0;
  bool keep = false;
  if (in) {
    const int n0 = n[b], a = adv[b];
    nn = n0 + a;
    keep = nn < T;
    my_kt = min(K, T - n0);
    my_adv = a;
    if (rej) my_rej = rej[b];
    n_new[b] = nn;
    id_all[b] = chain_id[b];
  }
  const unsigned long long m = __ballot(keep);
  const int before = __popcll(m & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = __popcll(m);
  __syncthreads();
  int offset = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kScanWaves; ++w) {
    const int c = wave_tot[w];
    offset += w < wave ? c : 0;
    total += c;
  }
  if (b < B) rank[b] = keep ? offset + before : (in ? -1 : -2);
  if (tid == 0) totals[blockIdx.x] = total;
  if (counters) {
    // wavefront sums first: one LDS atomic per wavefront and counter, one global atomic per workgroup
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
      my_adv += __shfl_xor(my_adv, s, 64);
      my_rej += __shfl_xor(my_rej, s, 64);
      my_kt += __shfl_xor(my_kt, s, 64);
    }
    if (lane == 0) {
      atomicAdd(reinterpret_cast<unsigned long long*>(&sh_cnt[0]), static_cast<unsigned long long>(my_adv));
      atomicAdd(reinterpret_cast<unsigned long long*>(&sh_cnt[2]), static_cast<unsigned long long>(my_rej));
      atomicAdd(reinterpret_cast<unsigned long long*>(&sh_cnt[1]), static_cast<unsigned long long>(my_kt));
    }
    __syncthreads();
    if (tid == 0) {
      unsigned long long* c = reinterpret_cast<unsigned long long*>(counters);
      if (sh_cnt[0]) atomicAdd(c + 0, static_cast<unsigned long long>(sh_cnt[0]));
      if (sh_cnt[2]) atomicAdd(c + 2, static_cast<unsigned long long>(sh_cnt[2]));
      if (sh_cnt[1]) atomicAdd(c + 4, static_cast<unsigned long long>(sh_cnt[1]));
      if (blockIdx.x == 0) {
        atomicAdd(c + 1, static_cast<unsigned long long>(Bact));
        atomicAdd(c + 3, Bact > 0 ? 1ull : 0ull);
      }
    }
  }
}

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

template <int VEC>
__global__ __launch_bounds__(kBlock) void advance_move_kernel(const float* __restrict__ y_out,
                                                              const int32_t* __restrict__ rank,
                                                              const int32_t* __restrict__ n_new,
                                                              const int64_t* __restrict__ id_all,
                                                              const int32_t* __restrict__ totals, float* __restrict__ y,
                                                              int32_t* __restrict__ n, int64_t* __restrict__ chain_id,
                                                              float* __restrict__ out, int32_t* __restrict__ B_active,
                                                              int Bprev, int d, int chunks,
                                                              const float* __restrict__ carry_src,
                                                              float* __restrict__ carry_dst,
                                                              const int32_t* __restrict__ adv, int rs,
                                                              const uint8_t* __restrict__ carry_rej) {
  // Bprev = number of chains that entered the window (host bound; rows beyond the device-side count carry
  // rank -2 and are skipped).  chunks > 0: a row takes `chunks` workgroups; chunks < 0: a workgroup takes
  // -chunks whole rows.
  const int nwg = (Bprev + kScanBlock - 1) / kScanBlock;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int tot = 0;
    for (int w = 0; w < nwg; ++w) tot += totals[w];
    *B_active = tot;
  }
  const int ncol = d / VEC;
  int b, col;
  if (chunks > 0) {
    b = blockIdx.x / chunks;
    col = (blockIdx.x % chunks) * kBlock + threadIdx.x;
  } else {
    const int rows = -chunks;
    const int slot = threadIdx.x / ncol;
    b = blockIdx.x * rows + slot;
    col = slot < rows ? static_cast<int>(threadIdx.x) - slot * ncol : ncol;
  }
  if (b >= Bprev) return;
  const int r = rank[b];
  if (r == -2) return;
  int dpos = -1;
  if (r >= 0) {
    dpos = r;
    const int wg = b / kScanBlock;
    for (int w = 0; w < wg; ++w) dpos += totals[w];
  }
  const int64_t id = id_all[b];
  if (dpos >= 0 && (chunks > 0 ? blockIdx.x % chunks == 0 && threadIdx.x == 0 : col == 0)) {
    n[dpos] = n_new[b];
    chain_id[dpos] = id;
  }
  float* dst = dpos >= 0 ? y + static_cast<int64_t>(dpos) * d : out + id * d;
  const float* src = y_out + static_cast<int64_t>(b) * d;
  if (col < ncol) {
    Pack<VEC> v;
    v.load(src + static_cast<int64_t>(col) * VEC);
    v.store(dst + static_cast<int64_t>(col) * VEC);
    if (carry_src && dpos >= 0) {
      // the surviving chain also takes along the next window's frozen vector: the target's prediction at the
      // draft state of the position it advanced to, or (carry_rej given) after a rejection the one at the last
      // state it kept, one row earlier
      const int row = adv[b] - (carry_rej && carry_rej[b] ? 1 : 0);
      v.load(carry_src + (static_cast<int64_t>(b) * rs + row) * d + static_cast<int64_t>(col) * VEC);
      v.store(carry_dst + static_cast<int64_t>(dpos) * d + static_cast<int64_t>(col) * VEC);
    }
  }
}

int check_ctx(sd_ctx* ctx) { return ctx ? SD_OK : SD_ERR_ARG; }

// ---------------------------------------------------------------------------------------------
// Scratch of sd_advance_static: the same layout sd_advance keeps in the caller's workspace (ids, ranks,
// new steps, survivor totals) for up to SD_STATIC_MAX_CHAINS chains, as a device array of the library
// itself.  Every GPU holds its own copy at its own address: sd_create resolves that address once per
// device (with the device current) and host code only ever uses the resolved pointer.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes =
    static_cast<size_t>(SD_STATIC_MAX_CHAINS) * 16 + (SD_STATIC_MAX_CHAINS / kScanBlock) * 4;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device.  Resolved on first use per device.
hipError_t static_scratch(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

template <int TPC, int VEC, int GROUPS>
void launch_verify(bool frozen, int B, hipStream_t st, const VerifyArgs& p) {
  constexpr int BLOCK = TPC > kBlock ? TPC : kBlock;
  constexpr int CPW = BLOCK / TPC;
  const unsigned grid = static_cast<unsigned>((B + CPW - 1) / CPW);
  if (frozen) hipLaunchKernelGGL((verify_kernel<TPC, VEC, true, GROUPS>), dim3(grid), dim3(BLOCK), 0, st, p);
  else        hipLaunchKernelGGL((verify_kernel<TPC, VEC, false, 0>), dim3(grid), dim3(BLOCK), 0, st, p);
}

// Launch shape by row length (ncol = 16-byte columns, or elements when the rows are not 16-byte aligned).
// Rows of more than 256 columns take (threads per chain, positions per group) from `shape`: 0 = the default
// for the row length, 1..4 = the alternatives it was measured against (sd_set_verify_shape).
template <int VEC>
void dispatch_verify(bool frozen, int B, int ncol, int shape, hipStream_t st, const VerifyArgs& p) {
  if (ncol <= 32) return launch_verify<16, VEC, 0>(frozen, B, st, p);
  if (ncol <= 256) return launch_verify<64, VEC, 0>(frozen, B, st, p);
  if (shape == 0) shape = ncol <= 1024 ? 2 : 4;
  switch (shape) {
    case 1: return launch_verify<256, VEC, 0>(frozen, B, st, p);
    case 2: return launch_verify<256, VEC, 1>(frozen, B, st, p);
    case 3: return launch_verify<512, VEC, 0>(frozen, B, st, p);
    default: return launch_verify<512, VEC, 1>(frozen, B, st, p);
  }
}

}  // namespace

// =============================================================================================
// C entry points
// =============================================================================================
extern "C" {

int sd_create(const sd_schedule* s, int32_t d, int32_t K, sd_ctx** out) {
  if (!s || !out || !s->a || !s->c || !s->sigma)
    return sdi::fail(g_create_error, SD_ERR_ARG, "sd_create: null argument");
  if (s->T <= 0 || d <= 0 || K <= 0 || K > SD_MAX_WINDOW)
    return sdi::fail(g_create_error, SD_ERR_ARG, "sd_create: need T>0, d>0, 1<=K<=%d (T=%d d=%d K=%d)",
                     SD_MAX_WINDOW, s->T, d, K);
  for (int k = 0; k < s->T; ++k) {
    if (!std::isfinite(s->a[k]) || !std::isfinite(s->c[k]) || !std::isfinite(s->sigma[k]))
      return sdi::fail(g_create_error, SD_ERR_SCHEDULE, "sd_create: non-finite coefficient at step %d", k);
    if (!(s->sigma[k] > 0.f))
      return sdi::fail(g_create_error, SD_ERR_SCHEDULE, "sd_create: sigma[%d]=%g must be > 0", k,
                       static_cast<double>(s->sigma[k]));
  }
  sd_ctx* ctx = new (std::nothrow) sd_ctx;
  if (!ctx) return sdi::fail(g_create_error, SD_ERR_ARG, "sd_create: out of host memory");
  ctx->T = s->T; ctx->d = d; ctx->K = K;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = static_scratch(ctx->device, &ctx->static_ws);   // this device's copy of the static scratch
  if (e == hipSuccess) e = sdi::langevin_prepare(&ctx->cus);
  float* dev = nullptr;
  const size_t sched_floats = (3 * static_cast<size_t>(s->T) + 15) / 16 * 16;   // counters start 64-byte aligned
  if (e == hipSuccess) e = hipMalloc(&dev, sizeof(float) * sched_floats + 64);
  if (e == hipSuccess) e = hipMemset(dev + sched_floats, 0, 64);
  if (e == hipSuccess) e = hipMemcpy(dev, s->a, sizeof(float) * s->T, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(dev + s->T, s->c, sizeof(float) * s->T, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(dev + 2 * s->T, s->sigma, sizeof(float) * s->T, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    if (dev) (void)hipFree(dev);
    delete ctx;
    return sdi::fail(g_create_error, SD_ERR_HIP, "sd_create: %s", hipGetErrorString(e));
  }
  ctx->dev_a = dev; ctx->dev_c = dev + s->T; ctx->dev_sigma = dev + 2 * s->T;
  ctx->dev_queue = reinterpret_cast<int32_t*>(dev + sched_floats);
  *out = ctx;
  return SD_OK;
}

int sd_destroy(sd_ctx* ctx) {
  if (!ctx) return SD_ERR_ARG;
  if (ctx->dev_a) (void)hipFree(ctx->dev_a);
  delete ctx;
  return SD_OK;
}

int sd_set_seed(sd_ctx* ctx, uint64_t seed) {
  if (!ctx) return SD_ERR_ARG;
  ctx->seed = seed;
  return SD_OK;
}

int sd_set_draft_mode(sd_ctx* ctx, int mode) {
  if (!ctx) return SD_ERR_ARG;
  if (mode != SD_DRAFT_FROZEN && mode != SD_DRAFT_EXPLICIT && mode != SD_DRAFT_FROZEN_REUSED)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_set_draft_mode: unknown mode %d", mode);
  ctx->mode = mode;
  return SD_OK;
}

int sd_set_temperature(sd_ctx* ctx, float tau) {
  if (!ctx) return SD_ERR_ARG;
  if (!(tau > 0.f) || !std::isfinite(tau))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_set_temperature: tau=%g must be finite and > 0",
                     static_cast<double>(tau));
  ctx->tau = tau;
  return SD_OK;
}

int sd_set_carry(sd_ctx* ctx, const float* Dq_ext, float* D_frozen) {
  if (!ctx) return SD_ERR_ARG;
  if ((Dq_ext == nullptr) != (D_frozen == nullptr))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_set_carry: give both arrays or neither");
  ctx->carry_src = Dq_ext;
  ctx->carry_dst = D_frozen;
  return SD_OK;
}

int sd_set_carry_rule(sd_ctx* ctx, int32_t rule) {
  if (!ctx) return SD_ERR_ARG;
  if (rule != SD_CARRY_DRAFT && rule != SD_CARRY_LAST_ACCEPTED)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_set_carry_rule: rule must be SD_CARRY_DRAFT or SD_CARRY_LAST_ACCEPTED");
  ctx->carry_rule = rule;
  return SD_OK;
}

int sd_set_draft_mirror(sd_ctx* ctx, uint16_t* Ytilde_bf16) {
  if (!ctx) return SD_ERR_ARG;
  ctx->draft_mirror = Ytilde_bf16;
  return SD_OK;
}

int sd_set_start_prediction(sd_ctx* ctx, const float* D_start) {
  if (!ctx) return SD_ERR_ARG;
  ctx->start_pred = D_start;
  return SD_OK;
}

int sd_set_verify_shape(sd_ctx* ctx, int32_t shape) {
  if (!ctx) return SD_ERR_ARG;
  if (shape < 0 || shape > 4) return sdi::fail(ctx->err, SD_ERR_ARG, "sd_set_verify_shape: shape must be 0..4");
  ctx->verify_shape = shape;
  return SD_OK;
}

int sd_set_active_count(sd_ctx* ctx, const int32_t* count) {
  if (!ctx) return SD_ERR_ARG;
  ctx->active = count;
  return SD_OK;
}

size_t sd_workspace_bytes(const sd_ctx* ctx, int32_t Bmax) {
  if (!ctx || Bmax <= 0) return 0;
  // ids int64[B], then rank int32[B], new steps int32[B], survivor totals int32[one per 1024 chains]
  const size_t b = static_cast<size_t>(Bmax);
  return b * 8 + b * 4 + b * 4 + ((b + kScanBlock - 1) / kScanBlock) * 4;
}

int sd_set_workspace(sd_ctx* ctx, void* workspace, size_t bytes) {
  if (!ctx) return SD_ERR_ARG;
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 7u))
    return sdi::fail(ctx->err, SD_ERR_WORKSPACE, "sd_set_workspace: buffer must be 8-byte aligned");
  ctx->ws = workspace;
  ctx->ws_bytes = workspace ? bytes : 0;
  return SD_OK;
}

int sd_init_state(sd_ctx* ctx, int32_t B, const int64_t* chain_id, float* y, int32_t* n, void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (B < 0 || (B > 0 && (!chain_id || !y || !n)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_init_state: bad argument");
  if (B == 0) return SD_OK;
  const int nblk = (ctx->d + 3) / 4;
  const int64_t total = static_cast<int64_t>(B) * nblk;
  const int64_t grid = (total + kBlock - 1) / kBlock;
  if (grid > 0x7fffffffLL) return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_init_state: B*d too large");
  hipLaunchKernelGGL(init_state_kernel, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0,
                     static_cast<hipStream_t>(stream), chain_id, y, n, B, ctx->d, nblk, ctx->seed);
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

int sd_draft(sd_ctx* ctx, int32_t B, const float* y, const int32_t* n, const int64_t* chain_id,
             const float* D0, float* Ytilde, int32_t* krow, void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (ctx->mode == SD_DRAFT_EXPLICIT)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_draft: only the frozen drafters are rolled out in one call; "
                                           "in EXPLICIT mode the caller produces the drafts and their means (sd_draft_step)");
  if (B < 0 || (B > 0 && (!y || !n || !chain_id || !D0 || !Ytilde || !krow)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_draft: bad argument");
  if (B == 0) return SD_OK;
  DraftArgs p;
  p.y = y; p.D0 = D0; p.n = n; p.id = chain_id; p.Ytil = Ytilde; p.krow = krow; p.mirror = ctx->draft_mirror;
  p.a = ctx->dev_a; p.c = ctx->dev_c; p.sigma = ctx->dev_sigma; p.active = ctx->active;
  p.B = B; p.d = ctx->d; p.K = ctx->K; p.T = ctx->T; p.nblk = (ctx->d + 3) / 4; p.seed = ctx->seed;
  const bool ext = ctx->mode == SD_DRAFT_FROZEN_REUSED;
  p.rs = ext ? ctx->K + 1 : ctx->K; p.roff = ext ? 1 : 0;
  const int64_t total = static_cast<int64_t>(B) * p.nblk;
  const int64_t grid = (total + kBlock - 1) / kBlock;
  if (grid > 0x7fffffffLL) return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_draft: B*d too large");
  const bool vec = (ctx->d % 4 == 0) && sdi::aligned16(y) && sdi::aligned16(D0) && sdi::aligned16(Ytilde) &&
                   sdi::aligned16(ctx->draft_mirror);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (vec) hipLaunchKernelGGL(draft_frozen_kernel<4>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st, p);
  else     hipLaunchKernelGGL(draft_frozen_kernel<1>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st, p);
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

int sd_draft_step(sd_ctx* ctx, int32_t B, int32_t j, const float* prev, const int32_t* n, const int64_t* chain_id,
                  const float* Dp, float* mp, float* Ytilde, int32_t* krow, float* next, int32_t* knext,
                  void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (B < 0 || j < 1 || j > ctx->K || (B > 0 && (!prev || !n || !chain_id || !Dp || !mp || !Ytilde || !krow)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_draft_step: bad argument (j must be in 1..K)");
  if (next && (next == prev || next == Dp))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_draft_step: next must not alias prev or Dp");
  if (B == 0) return SD_OK;
  DraftStepArgs p;
  p.prev = prev; p.Dp = Dp; p.n = n; p.id = chain_id; p.mp = mp; p.Ytil = Ytilde; p.next = next;
  p.krow = krow; p.knext = knext;
  p.a = ctx->dev_a; p.c = ctx->dev_c; p.sigma = ctx->dev_sigma; p.active = ctx->active;
  p.B = B; p.d = ctx->d; p.K = ctx->K; p.T = ctx->T; p.nblk = (ctx->d + 3) / 4; p.j = j; p.seed = ctx->seed;
  const int64_t total = static_cast<int64_t>(B) * p.nblk;
  const int64_t grid = (total + kBlock - 1) / kBlock;
  if (grid > 0x7fffffffLL) return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_draft_step: B*d too large");
  const bool vec = (ctx->d % 4 == 0) && sdi::aligned16(prev) && sdi::aligned16(Dp) && sdi::aligned16(mp) &&
                   sdi::aligned16(Ytilde) && sdi::aligned16(next);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (vec) hipLaunchKernelGGL(draft_step_kernel<4>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st, p);
  else     hipLaunchKernelGGL(draft_step_kernel<1>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st, p);
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

int sd_verify(sd_ctx* ctx, int32_t B, const float* y, const int32_t* n, const int64_t* chain_id,
              const float* D0_or_mp, const float* Dq, const float* Ytilde, float* y_out,
              int32_t* adv, uint8_t* rejected, float* logratio, float* logu, void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (B < 0 || (B > 0 && (!y || !n || !chain_id || !D0_or_mp || !Dq || !Ytilde || !y_out || !adv)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_verify: bad argument");
  if (B == 0) return SD_OK;
  VerifyArgs p;
  p.y = y; p.D0mp = D0_or_mp; p.Dq = Dq; p.Ytil = Ytilde; p.n = n; p.id = chain_id;
  p.y_out = y_out; p.adv = adv; p.rej = rejected; p.logratio = logratio; p.logu = logu;
  p.Dq0 = ctx->mode == SD_DRAFT_EXPLICIT ? ctx->start_pred : nullptr;
  const bool ext = ctx->mode == SD_DRAFT_FROZEN_REUSED;
  p.rs = ext ? ctx->K + 1 : ctx->K; p.roff = ext ? 1 : 0; p.first_exact = ctx->mode == SD_DRAFT_FROZEN;
  p.a = ctx->dev_a; p.c = ctx->dev_c; p.sigma = ctx->dev_sigma; p.active = ctx->active;
  p.B = B; p.d = ctx->d; p.K = ctx->K; p.T = ctx->T; p.seed = ctx->seed; p.inv_tau = 1.0 / ctx->tau;
  const bool frozen = ctx->mode != SD_DRAFT_EXPLICIT;
  const bool vec = (ctx->d % 4 == 0) && sdi::aligned16(y) && sdi::aligned16(D0_or_mp) && sdi::aligned16(p.Dq0) &&
                   sdi::aligned16(Dq) && sdi::aligned16(Ytilde) && sdi::aligned16(y_out);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int ncol = vec ? ctx->d / 4 : ctx->d;
  if (vec) dispatch_verify<4>(frozen, B, ncol, ctx->verify_shape, st, p);
  else     dispatch_verify<1>(frozen, B, ncol, ctx->verify_shape, st, p);
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

}  // extern "C"

// Both advance entry points: `ws` holds sd_workspace_bytes(ctx, B) bytes of device scratch.
static int advance_impl(sd_ctx* ctx, void* ws, int32_t B, const float* y_out, const int32_t* adv,
                        const uint8_t* rejected, float* y, int32_t* n, int64_t* chain_id, float* out,
                        int32_t* B_active, int64_t* counters, hipStream_t st) {
  if (ctx->mode == SD_DRAFT_FROZEN_REUSED && ctx->carry_src && ctx->carry_rule == SD_CARRY_LAST_ACCEPTED && !rejected)
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_advance: the last-accepted carry rule needs the `rejected` array");
  if (B == 0) {
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, st, B_active, 0);
    SD_HIP_TRY(ctx->err, hipGetLastError());
    return SD_OK;
  }
  int64_t* id_all = static_cast<int64_t*>(ws);
  int32_t* rank = reinterpret_cast<int32_t*>(id_all + B);
  int32_t* n_new = rank + B;
  int32_t* totals = n_new + B;
  const int nwg = (B + kScanBlock - 1) / kScanBlock;
  hipLaunchKernelGGL(advance_rank_kernel, dim3(nwg), dim3(kScanBlock), 0, st, adv, rejected, n, chain_id, rank, n_new,
                     id_all, totals, counters, ctx->active, B, ctx->T, ctx->K);
  {
    const bool vec = (ctx->d % 4 == 0) && sdi::aligned16(y_out) && sdi::aligned16(y) && sdi::aligned16(out) &&
                     sdi::aligned16(ctx->carry_src) && sdi::aligned16(ctx->carry_dst);
    const int ncol = vec ? ctx->d / 4 : ctx->d;
    // short rows share a workgroup (negative `chunks` = rows per workgroup), long rows are split over several
    const int rows_per_wg = ncol <= kBlock / 2 ? kBlock / ncol : 1;
    const int chunks = rows_per_wg > 1 ? -rows_per_wg : (ncol + kBlock - 1) / kBlock;
    const int64_t grid = rows_per_wg > 1 ? (static_cast<int64_t>(B) + rows_per_wg - 1) / rows_per_wg
                                         : static_cast<int64_t>(B) * chunks;
    if (grid > 0x7fffffffLL) return sdi::fail(ctx->err, SD_ERR_UNSUPPORTED, "sd_advance: B*d too large");
    const float* csrc = ctx->mode == SD_DRAFT_FROZEN_REUSED ? ctx->carry_src : nullptr;
    const uint8_t* crej = csrc && ctx->carry_rule == SD_CARRY_LAST_ACCEPTED ? rejected : nullptr;
    if (vec) hipLaunchKernelGGL(advance_move_kernel<4>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st,
                                y_out, rank, n_new, id_all, totals, y, n, chain_id, out, B_active, B, ctx->d, chunks,
                                csrc, ctx->carry_dst, adv, ctx->K + 1, crej);
    else     hipLaunchKernelGGL(advance_move_kernel<1>, dim3(static_cast<unsigned>(grid)), dim3(kBlock), 0, st,
                                y_out, rank, n_new, id_all, totals, y, n, chain_id, out, B_active, B, ctx->d, chunks,
                                csrc, ctx->carry_dst, adv, ctx->K + 1, crej);
  }
  SD_HIP_TRY(ctx->err, hipGetLastError());
  return SD_OK;
}

extern "C" {

int sd_advance(sd_ctx* ctx, int32_t B, const float* y_out, const int32_t* adv, const uint8_t* rejected,
               float* y, int32_t* n, int64_t* chain_id, float* out, int32_t* B_active,
               int64_t* counters, void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (B < 0 || !B_active || (B > 0 && (!y_out || !adv || !y || !n || !chain_id || !out)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_advance: bad argument");
  if (B > 0 && (!ctx->ws || ctx->ws_bytes < sd_workspace_bytes(ctx, B)))
    return sdi::fail(ctx->err, SD_ERR_WORKSPACE, "sd_advance: workspace of %zu bytes needed for B=%d, have %zu",
                     sd_workspace_bytes(ctx, B), B, ctx->ws_bytes);
  return advance_impl(ctx, ctx->ws, B, y_out, adv, rejected, y, n, chain_id, out, B_active, counters,
                      static_cast<hipStream_t>(stream));
}

int sd_advance_static(sd_ctx* ctx, int32_t B, const float* y_out, const int32_t* adv, const uint8_t* rejected,
                      float* y, int32_t* n, int64_t* chain_id, float* out, int32_t* B_active,
                      int64_t* counters, void* stream) {
  if (int rc = check_ctx(ctx)) return rc;
  if (B < 0 || !B_active || (B > 0 && (!y_out || !adv || !y || !n || !chain_id || !out)))
    return sdi::fail(ctx->err, SD_ERR_ARG, "sd_advance_static: bad argument");
  if (B > SD_STATIC_MAX_CHAINS)
    return sdi::fail(ctx->err, SD_ERR_WORKSPACE, "sd_advance_static: B=%d exceeds the %d chains the static scratch holds "
                                                 "(use sd_advance with a workspace)", B, SD_STATIC_MAX_CHAINS);
  if (!ctx->static_ws)
    return sdi::fail(ctx->err, SD_ERR_HIP, "sd_advance_static: the static scratch was not resolved at sd_create");
  return advance_impl(ctx, ctx->static_ws, B, y_out, adv, rejected, y, n, chain_id, out, B_active, counters,
                      static_cast<hipStream_t>(stream));
}

const char* sd_last_error(const sd_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
