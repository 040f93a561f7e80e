// Counter-based random streams of the chains, device side.
//
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) with
//   key     = (seed low word, seed high word)
//   counter = (chain_id low, chain_id high, state index k, (stream << 28) | block)
// One block = four 32-bit words = elements 4*block .. 4*block+3 of a d-vector.
// word -> uniform u = ((w >> 9) + 1/2) * 2^-23 (exact in fp32, strictly inside (0,1));
// words (0,1) and (2,3) -> two Box-Muller pairs  r (cos, sin)(2 pi u_odd), r = sqrt(-2 ln u_even).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace sdrng {

constexpr uint32_t kStreamNoise = 0u;
constexpr uint32_t kStreamUniform = 1u;
constexpr uint32_t kStreamInit = 2u;

struct Words {
  uint32_t w[4];
};

__device__ __forceinline__ Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Words{{c0, c1, c2, c3}};
}

__device__ __forceinline__ Words block_words(uint64_t seed, int64_t chain_id, uint32_t k,
                                             uint32_t stream, uint32_t block) {
  const uint64_t id = static_cast<uint64_t>(chain_id);
  return philox4x32_10(static_cast<uint32_t>(id), static_cast<uint32_t>(id >> 32), k,
                       (stream << 28) | block, static_cast<uint32_t>(seed),
                       static_cast<uint32_t>(seed >> 32));
}

__device__ __forceinline__ float word_to_uniform(uint32_t w) {
  return (static_cast<float>(w >> 9) + 0.5f) * 0x1p-23f;
}

__device__ __forceinline__ void box_muller(uint32_t w_even, uint32_t w_odd, float& z_even,
                                           float& z_odd) {
  // hardware transcendentals: log2, sqrt (1 ulp) and sine / cosine of an angle given in turns, which is what
  // the uniform already is (no range reduction).  Measured over all 2^23 uniforms against fp64: radius within
  // 1.4e-7 relative (the library's logf / sqrtf: 1.5e-7), sine and cosine within 1.3e-7 absolute (sincospif:
  // 0.5e-7), at a third of the instructions.
  const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(word_to_uniform(w_even)));
  const float turn = word_to_uniform(w_odd);
  z_even = r * __builtin_amdgcn_cosf(turn);
  z_odd = r * __builtin_amdgcn_sinf(turn);
}

// Four standard normals: elements 4*block .. 4*block+3 of the vector keyed (chain_id, k, stream).
__device__ __forceinline__ void normal4(uint64_t seed, int64_t chain_id, uint32_t k,
                                        uint32_t stream, uint32_t block, float z[4]) {
  const Words w = block_words(seed, chain_id, k, stream, block);
  box_muller(w.w[0], w.w[1], z[0], z[1]);
  box_muller(w.w[2], w.w[3], z[2], z[3]);
}

// log of the accept-test uniform of state k, in fp64 (it is compared with an fp64 log-ratio).
__device__ __forceinline__ double log_uniform(uint64_t seed, int64_t chain_id, uint32_t k) {
  const Words w = block_words(seed, chain_id, k, kStreamUniform, 0u);
  return log(static_cast<double>(word_to_uniform(w.w[0])));
}

}  // namespace sdrng
