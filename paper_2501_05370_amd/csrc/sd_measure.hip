// Measurement kernels: what plain streaming and a loop of nothing but MFMAs reach on this chip
// (the ceilings the hot-path kernels are compared with next to the published peaks).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/sd.h"
#include "../../include/sd_measure.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

int compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  return cus;
}

template <int MODE>
__global__ __launch_bounds__(256) void stream_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (MODE == 0) {
    // four accesses in flight per thread
    for (; i + 3 * stride < n16; i += 4 * stride) {
      const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
      dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
  } else if (MODE == 1) {
    float acc = 0.f;
    for (; i + 3 * stride < n16; i += 4 * stride) {
      const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
      acc += (a.x + a.y + a.z + a.w) + (b.x + b.y + b.z + b.w) + (c.x + c.y + c.z + c.w) + (d.x + d.y + d.z + d.w);
    }
    for (; i < n16; i += stride) {
      const float4 a = src[i];
      acc += a.x + a.y + a.z + a.w;
    }
    __shared__ float sh[256];
    sh[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.f;
      for (int k = 0; k < 256; ++k) t += sh[k];
      reinterpret_cast<float*>(dst)[blockIdx.x] = t;
    }
  } else {
    const float4 v = make_float4(1.f, 2.f, 3.f, 4.f);
    for (; i < n16; i += stride) dst[i] = v;
  }
}

// The same three passes with the access pattern of the window kernels: a workgroup takes whole rows of kRowBytes
// (the 48 KiB of a 12288-wide fp32 row), row after row, each thread requesting all its 16-byte pieces of the row
// before it uses any.
constexpr int kRowBytes = 49152;
template <int MODE>
__global__ __launch_bounds__(256) void stream_rows_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t nrows) {
  constexpr int PER = kRowBytes / 16 / 256;        // 12 pieces per thread and row
  float acc = 0.f;
  for (size_t r = blockIdx.x; r < nrows; r += gridDim.x) {
    const size_t base = r * (kRowBytes / 16) + threadIdx.x;
    if (MODE == 2) {
      const float4 v = make_float4(1.f, 2.f, 3.f, 4.f);
#pragma unroll
      for (int i = 0; i < PER; ++i) dst[base + i * 256] = v;
    } else {
      float4 v[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) v[i] = src[base + i * 256];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        if (MODE == 0) dst[base + i * 256] = v[i];
        else acc += v[i].x + v[i].y + v[i].z + v[i].w;
      }
    }
  }
  if (MODE == 1) {
    __shared__ float sh[256];
    sh[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.f;
      for (int k = 0; k < 256; ++k) t += sh[k];
      reinterpret_cast<float*>(dst)[blockIdx.x] = t;
    }
  }
}

template <int SHAPE>
__global__ __launch_bounds__(512) void mfma_kernel(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = static_cast<__bf16>(0.001f * static_cast<float>((lane * 7 + e * 3) % 13 - 6));
    b[e] = static_cast<__bf16>(0.001f * static_cast<float>((lane * 5 + e) % 11 - 5));
  }
  float total = 0.f;
  if (SHAPE == 0) {
    f32x16 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) total += acc[t][v];
  } else {
    f32x4 acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 16; ++t) total += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
  }
  if (total == 12345.678f) sink[blockIdx.x] = total;      // keeps the accumulators alive; practically never taken
  if (threadIdx.x == 0 && iters == 0) sink[blockIdx.x] = total;
}

}  // namespace

extern "C" {

int sd_measure_stream(const void* src, void* dst, size_t bytes, int32_t mode, int32_t workgroups, void* stream) {
  const bool by_rows = mode >= 3;
  if (by_rows) mode -= 3;
  if (by_rows && bytes % kRowBytes != 0) return SD_ERR_ARG;
  if (!dst || (mode != 2 && !src) || bytes == 0 || (bytes & 15u) || mode < 0 || mode > 2 || workgroups < 0 ||
      workgroups > 4096 || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u))
    return SD_ERR_ARG;
  const int grid = workgroups > 0 ? workgroups : 16 * compute_units();
  if (grid > 4096) return SD_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const float4* s = static_cast<const float4*>(src);
  float4* d = static_cast<float4*>(dst);
  if (by_rows) {
    const size_t nrows = bytes / kRowBytes;
    if (mode == 0) hipLaunchKernelGGL(stream_rows_kernel<0>, dim3(grid), dim3(256), 0, st, s, d, nrows);
    else if (mode == 1) hipLaunchKernelGGL(stream_rows_kernel<1>, dim3(grid), dim3(256), 0, st, s, d, nrows);
    else hipLaunchKernelGGL(stream_rows_kernel<2>, dim3(grid), dim3(256), 0, st, s, d, nrows);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
  }
  if (mode == 0) hipLaunchKernelGGL(stream_kernel<0>, dim3(grid), dim3(256), 0, st, s, d, bytes / 16);
  else if (mode == 1) hipLaunchKernelGGL(stream_kernel<1>, dim3(grid), dim3(256), 0, st, s, d, bytes / 16);
  else hipLaunchKernelGGL(stream_kernel<2>, dim3(grid), dim3(256), 0, st, s, d, bytes / 16);
  return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

int sd_measure_mfma(int32_t shape, int32_t iters, int32_t workgroups, float* sink, double* flops, void* stream) {
  if (!sink || shape < 0 || shape > 1 || iters < 0 || workgroups < 0 || workgroups > 65536) return SD_ERR_ARG;
  const int grid = workgroups > 0 ? workgroups : compute_units();
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (shape == 0) hipLaunchKernelGGL(mfma_kernel<0>, dim3(grid), dim3(512), 0, st, iters, sink);
  else hipLaunchKernelGGL(mfma_kernel<1>, dim3(grid), dim3(512), 0, st, iters, sink);
  // 16 MFMAs per round and wavefront, 8 wavefronts per workgroup
  if (flops) *flops = static_cast<double>(grid) * 8.0 * iters * 16.0 * (shape == 0 ? 32768.0 : 16384.0);
  return hipGetLastError() == hipSuccess ? SD_OK : SD_ERR_HIP;
}

}  // extern "C"
