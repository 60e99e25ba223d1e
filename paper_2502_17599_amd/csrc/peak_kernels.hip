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

// Four independent accumulator chains per wave, eight operand pairs per wave held in registers; one workgroup =
// one wave per SIMD, two workgroups per CU.  Nothing is loaded; the sum of the accumulators is stored under a
// condition that is false for these operands.  The operands are either nearly constant (bf16 values near 1,
// the same in most lanes) or pseudo-random (sign, mantissa and the lowest exponent bit vary from lane to lane and
// from step to step): the matrix unit's power draw, and with it the clock the chip can hold, depends on how many
// operand bits toggle, so the two give different rates.
__global__ void __launch_bounds__(kPeakThreads, 2) peak_mfma_bf16_kernel(long long rounds, int random_operands, float* sink) {
  const uint32_t seed = 0x3f803f80u + (threadIdx.x & 7u);  // pairs of bf16 values near 1
  uint4 a4[8], b4[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a4[i] = make_uint4(seed, seed ^ 0x00010000u, seed, seed ^ 0x00000001u);
    b4[i] = make_uint4(seed ^ 0x00020002u, seed, seed ^ 0x00010001u, seed);
  }
  if (random_operands) {
    uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    auto word = [&]() {  // two bf16 values of magnitude 0.5 .. 2 with random sign and mantissa
      h = h * 1664525u + 1013904223u;
      const uint32_t v = h >> 8;
      return ((v & 0x80ffu) | 0x3f00u) | ((((v >> 12) & 0x80ffu) | 0x3f00u) << 16);
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a4[i] = make_uint4(word(), word(), word(), word());
      b4[i] = make_uint4(word(), word(), word(), word());
    }
  }
  f32x16_t c0 = acc_zero(), c1 = acc_zero(), c2 = acc_zero(), c3 = acc_zero();
  for (long long r = 0; r < rounds; ++r) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bf16x8_t a = __builtin_bit_cast(bf16x8_t, a4[(2 * u) & 7]), b = __builtin_bit_cast(bf16x8_t, b4[(2 * u) & 7]);
      const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, a4[(2 * u + 1) & 7]), b2 = __builtin_bit_cast(bf16x8_t, b4[(2 * u + 1) & 7]);
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b2, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b2, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, b, c3, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.0f) *sink = s;
}

// How much vector work fits beside the matrix instructions: every round issues 16 matrix instructions (two
// accumulator chains) and 16 * V independent fp32 multiply-adds on private registers, the multiply-adds either
// right behind each matrix instruction (INTERLEAVED; the order is pinned with a scheduling barrier per pair of
// matrix instructions) or all after the sixteenth (a matrix phase and a vector phase, as a kernel has them whose
// vector work depends on the products).  Nearly constant operands, no memory.  The multiply-adds are volatile asm
// so that they are neither merged nor moved.
template <int V, bool INTERLEAVED>
__global__ void __launch_bounds__(kPeakThreads, 2) peak_mfma_valu_kernel(long long rounds, float* sink) {
  const uint32_t seed = 0x3f803f80u + (threadIdx.x & 7u);
  const uint4 a4 = make_uint4(seed, seed ^ 0x00010000u, seed, seed ^ 0x00000001u);
  const uint4 b4 = make_uint4(seed ^ 0x00020002u, seed, seed ^ 0x00010001u, seed);
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, a4), b = __builtin_bit_cast(bf16x8_t, b4);
  f32x16_t c0 = acc_zero(), c1 = acc_zero();
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 1.0f + threadIdx.x * 1e-3f + i;
  const float m = 0.999f, d = 1e-3f;  // x stays bounded: x <- 0.999 x + 0.001
  for (long long r = 0; r < rounds; ++r) {
    if constexpr (INTERLEAVED) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < V; ++j) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[j & 7]) : "v"(m), "v"(d));
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c1, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < V; ++j) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[(j + 4) & 7]) : "v"(m), "v"(d));
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c1, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < 16 * V; ++j) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[j & 7]) : "v"(m), "v"(d));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i];
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
  if (s == -1.0f) *sink = s;
}

template <bool INTERLEAVED>
static bool launch_mfma_valu(int v, unsigned blocks, long long rounds, float* sink, hipStream_t s) {
  switch (v) {
    case 0: hipLaunchKernelGGL((peak_mfma_valu_kernel<0, INTERLEAVED>), dim3(blocks), dim3(kPeakThreads), 0, s, rounds, sink); return true;
    case 4: hipLaunchKernelGGL((peak_mfma_valu_kernel<4, INTERLEAVED>), dim3(blocks), dim3(kPeakThreads), 0, s, rounds, sink); return true;
    case 6: hipLaunchKernelGGL((peak_mfma_valu_kernel<6, INTERLEAVED>), dim3(blocks), dim3(kPeakThreads), 0, s, rounds, sink); return true;
    case 8: hipLaunchKernelGGL((peak_mfma_valu_kernel<8, INTERLEAVED>), dim3(blocks), dim3(kPeakThreads), 0, s, rounds, sink); return true;
    default: return false;
  }
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

meda_status meda_peak_mfma_bf16(int64_t mfma_per_wave, int32_t random_operands, int64_t* total_mfma, void* sink,
                                void* hip_stream) {
  if (mfma_per_wave < 16 || mfma_per_wave > (1ll << 30) || !total_mfma || !sink || ((uintptr_t)sink & 3u))
    return MEDA_ERR_INVALID_ARG;
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess) return MEDA_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MEDA_ERR_HIP;
  const long long rounds = mfma_per_wave / 16;  // 16 matrix instructions per round
  const unsigned blocks = (unsigned)cus * 2u;   // two waves per SIMD
  hipLaunchKernelGGL(meda::peak_mfma_bf16_kernel, dim3(blocks), dim3(meda::kPeakThreads), 0,
                     static_cast<hipStream_t>(hip_stream), rounds, random_operands ? 1 : 0, static_cast<float*>(sink));
  if (hipGetLastError() != hipSuccess) return MEDA_ERR_HIP;
  *total_mfma = (int64_t)rounds * 16 * (meda::kPeakThreads / 64) * blocks;
  return MEDA_OK;
}

meda_status meda_peak_mfma_valu(int64_t rounds, int32_t valu_per_mfma, int32_t interleaved, int32_t waves_per_simd,
                                void* sink, void* hip_stream) {
  if (rounds < 1 || rounds > (1ll << 22) || !sink || ((uintptr_t)sink & 3u)) return MEDA_ERR_INVALID_ARG;
  if (valu_per_mfma != 0 && valu_per_mfma != 4 && valu_per_mfma != 6 && valu_per_mfma != 8) return MEDA_ERR_INVALID_ARG;
  if (waves_per_simd != 1 && waves_per_simd != 2) return MEDA_ERR_INVALID_ARG;
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess) return MEDA_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MEDA_ERR_HIP;
  const unsigned blocks = (unsigned)cus * (unsigned)waves_per_simd;  // a workgroup is one wave on every SIMD of a CU
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  float* snk = static_cast<float*>(sink);
  const bool ok = interleaved ? meda::launch_mfma_valu<true>(valu_per_mfma, blocks, rounds, snk, s)
                              : meda::launch_mfma_valu<false>(valu_per_mfma, blocks, rounds, snk, s);
  if (!ok) return MEDA_ERR_INVALID_ARG;
  return hipGetLastError() == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

}  // extern "C"
