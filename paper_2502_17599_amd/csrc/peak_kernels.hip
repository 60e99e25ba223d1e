// Measurement aids: the rates this GPU delivers to the simplest kernels of the two kinds the compression pass
// is made of -- a stream of 16-byte reads over a large buffer (what bounds the scoring and merge phases) and
// back-to-back bf16 32x32x16 matrix instructions out of registers (what bounds the similarity phase).  The
// benchmark prints both next to the published peaks; the roofline fractions stay priced against the published
// ones.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/meda.h"
#include "device_utils.hpp"

namespace meda {

constexpr int kPeakThreads = 256;
constexpr int kPeakReadsInFlight = 8;

// Every thread reads 16-byte pieces with a grid stride, eight loads in flight; the pieces are folded into one
// word that is stored only if it has a value the fold cannot produce twice in a row (keeps the loads alive).
__global__ void __launch_bounds__(kPeakThreads) peak_stream_read_kernel(const uint4* src, size_t n_pieces, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * kPeakThreads;
  size_t i = (size_t)blockIdx.x * kPeakThreads + threadIdx.x;
  uint32_t acc = 0;
  for (; i + (kPeakReadsInFlight - 1) * stride < n_pieces; i += kPeakReadsInFlight * stride) {
    uint4 v[kPeakReadsInFlight];
#pragma unroll
    for (int u = 0; u < kPeakReadsInFlight; ++u) v[u] = load16_stream(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < kPeakReadsInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n_pieces; i += stride) {
    const uint4 v = load16_stream(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) *sink = acc;
}

// Four independent accumulator chains per wave, operands made up from the lane id; one workgroup = one wave per
// SIMD, two workgroups per CU.  Nothing is loaded; the sum of the accumulators is stored under a condition that
// is false for these operands.
__global__ void __launch_bounds__(kPeakThreads, 2) peak_mfma_bf16_kernel(long long rounds, float* sink) {
  const uint32_t seed = 0x3f803f80u + (threadIdx.x & 7u);  // pairs of bf16 values near 1
  const uint4 a4 = make_uint4(seed, seed ^ 0x00010000u, seed, seed ^ 0x00000001u);
  const uint4 b4 = make_uint4(seed ^ 0x00020002u, seed, seed ^ 0x00010001u, seed);
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, a4), b = __builtin_bit_cast(bf16x8_t, b4);
  f32x16_t c0 = acc_zero(), c1 = acc_zero(), c2 = acc_zero(), c3 = acc_zero();
  for (long long r = 0; r < rounds; ++r) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.0f) *sink = s;
}

}  // namespace meda

extern "C" {

meda_status meda_peak_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 3u)) return MEDA_ERR_INVALID_ARG;
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess) return MEDA_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MEDA_ERR_HIP;
  const size_t n_pieces = bytes / 16;
  size_t blocks = (size_t)cus * 8;  // eight workgroups of four waves per CU
  const size_t needed = (n_pieces + meda::kPeakThreads - 1) / meda::kPeakThreads;
  if (blocks > needed) blocks = needed;
  hipLaunchKernelGGL(meda::peak_stream_read_kernel, dim3((unsigned)blocks), dim3(meda::kPeakThreads), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(src), n_pieces,
                     static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

meda_status meda_peak_mfma_bf16(int64_t mfma_per_wave, int64_t* total_mfma, void* sink, void* hip_stream) {
  if (mfma_per_wave < 16 || mfma_per_wave > (1ll << 30) || !total_mfma || !sink || ((uintptr_t)sink & 3u))
    return MEDA_ERR_INVALID_ARG;
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess) return MEDA_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MEDA_ERR_HIP;
  const long long rounds = mfma_per_wave / 16;  // 16 matrix instructions per round
  const unsigned blocks = (unsigned)cus * 2u;   // two waves per SIMD
  hipLaunchKernelGGL(meda::peak_mfma_bf16_kernel, dim3(blocks), dim3(meda::kPeakThreads), 0,
                     static_cast<hipStream_t>(hip_stream), rounds, static_cast<float*>(sink));
  if (hipGetLastError() != hipSuccess) return MEDA_ERR_HIP;
  *total_mfma = (int64_t)rounds * 16 * (meda::kPeakThreads / 64) * blocks;
  return MEDA_OK;
}

}  // extern "C"
