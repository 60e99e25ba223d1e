// Row-wise 8-bit storage of a compressed cache: quantiser and its inverse.  The paper names KV-cache
// quantisation as combinable with its method (Limitations section) and fixes no scheme; the scheme is this
// library's (per row: scale = max|x| / 448, codes in E4M3).  Both kernels stream rows once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/meda.h"
#include "device_utils.hpp"
#include "fp8.hpp"

namespace meda {

template <typename T>
struct RowPiece;   // the 16 bytes of a row one lane handles
template <>
struct RowPiece<bf16_t> {
  static constexpr int kElems = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
    uint4 o;
    o.x = float_to_bf16_rne(f[0]) | (float_to_bf16_rne(f[1]) << 16);
    o.y = float_to_bf16_rne(f[2]) | (float_to_bf16_rne(f[3]) << 16);
    o.z = float_to_bf16_rne(f[4]) | (float_to_bf16_rne(f[5]) << 16);
    o.w = float_to_bf16_rne(f[6]) | (float_to_bf16_rne(f[7]) << 16);
    return o;
  }
};
template <>
struct RowPiece<float> {
  static constexpr int kElems = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};

// LPR = D / E lanes read one row (16 bytes each); a wave takes 64 / LPR rows per step, grid-stride over the rows.
template <typename T, int D>
__global__ void __launch_bounds__(256) quantize_fp8_kernel(const char* rows, long long n_rows, uint8_t* codes,
                                                           float* scales) {
  using RP = RowPiece<T>;
  constexpr int E = RP::kElems, LPR = D / E, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane / LPR, cc = lane - sub * LPR;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long n_waves = ((long long)gridDim.x * blockDim.x) >> 6;
  for (long long r0 = wave * RPW; r0 < n_rows; r0 += n_waves * RPW) {
    const long long r = r0 + sub;
    const bool ok = r < n_rows;
    const long long rr = ok ? r : n_rows - 1;   // lanes past the end repeat the last row and store nothing
    const uint4 v = load16_stream(rows + ((size_t)rr * D + cc * E) * sizeof(T));
    float f[E];
    RP::unpack(v, f);
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
    for (int x = 1; x < LPR; x <<= 1) amax = fmaxf(amax, __shfl_xor(amax, x, kWave));
    const float scale = amax > 0.f ? amax / kE4M3Max : 1.0f;
    uint32_t w[(E + 3) / 4] = {0};
#pragma unroll
    for (int i = 0; i < E; ++i) {
      const float y = fminf(fmaxf(f[i] / scale, -kE4M3Max), kE4M3Max);
      w[i / 4] |= float_to_e4m3(y) << (8 * (i % 4));
    }
    if (ok) {
      uint8_t* dst = codes + (size_t)r * D + cc * E;
      if constexpr (E == 8) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
      else *reinterpret_cast<uint32_t*>(dst) = w[0];
      if (cc == 0) scales[r] = scale;
    }
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(256) dequantize_fp8_kernel(const uint8_t* codes, const float* scales,
                                                             long long n_rows, char* rows) {
  using RP = RowPiece<T>;
  constexpr int E = RP::kElems, LPR = D / E, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane / LPR, cc = lane - sub * LPR;
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const long long n_waves = ((long long)gridDim.x * blockDim.x) >> 6;
  for (long long r0 = wave * RPW; r0 < n_rows; r0 += n_waves * RPW) {
    const long long r = r0 + sub;
    if (r >= n_rows) continue;
    const uint8_t* src = codes + (size_t)r * D + cc * E;
    const float scale = scales[r];
    float f[E];
    if constexpr (E == 8) {
      const uint2 c = *reinterpret_cast<const uint2*>(src);
      e4m3x2_to_float(c.x, false, f[0], f[1]);
      e4m3x2_to_float(c.x, true, f[2], f[3]);
      e4m3x2_to_float(c.y, false, f[4], f[5]);
      e4m3x2_to_float(c.y, true, f[6], f[7]);
    } else {
      const uint32_t c = *reinterpret_cast<const uint32_t*>(src);
      e4m3x2_to_float(c, false, f[0], f[1]);
      e4m3x2_to_float(c, true, f[2], f[3]);
    }
#pragma unroll
    for (int i = 0; i < E; ++i) f[i] *= scale;
    *reinterpret_cast<uint4*>(rows + ((size_t)r * D + cc * E) * sizeof(T)) = RP::pack(f);
  }
}

static unsigned stream_grid(long long n_rows, int rows_per_wave) {
  const long long waves = (n_rows + rows_per_wave - 1) / rows_per_wave;
  long long blocks = (waves + 3) / 4;
  if (blocks > 256 * 16) blocks = 256 * 16;   // 16 workgroups per CU keep the loads of a grid-stride loop in flight
  return (unsigned)(blocks < 1 ? 1 : blocks);
}

}  // namespace meda

extern "C" {

meda_status meda_quantize_fp8(const void* rows, int32_t dtype, int64_t n_rows, int32_t head_dim, uint8_t* codes,
                              float* scales, void* hip_stream) {
  using namespace meda;
  if (n_rows < 0) return MEDA_ERR_INVALID_ARG;
  if (dtype != MEDA_F32 && dtype != MEDA_BF16) return MEDA_ERR_UNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return MEDA_ERR_UNSUPPORTED;
  if (n_rows == 0) return MEDA_OK;
  if (!rows || !codes || !scales) return MEDA_ERR_INVALID_ARG;
  if (((uintptr_t)rows | (uintptr_t)codes) & 15u || ((uintptr_t)scales & 3u)) return MEDA_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const char* src = static_cast<const char*>(rows);
  const int lpr = dtype == MEDA_BF16 ? head_dim / 8 : head_dim / 4;
  const dim3 grid(stream_grid(n_rows, 64 / lpr)), block(256);
  if (dtype == MEDA_BF16) {
    if (head_dim == 128) hipLaunchKernelGGL((quantize_fp8_kernel<bf16_t, 128>), grid, block, 0, s, src, (long long)n_rows, codes, scales);
    else hipLaunchKernelGGL((quantize_fp8_kernel<bf16_t, 64>), grid, block, 0, s, src, (long long)n_rows, codes, scales);
  } else {
    if (head_dim == 128) hipLaunchKernelGGL((quantize_fp8_kernel<float, 128>), grid, block, 0, s, src, (long long)n_rows, codes, scales);
    else hipLaunchKernelGGL((quantize_fp8_kernel<float, 64>), grid, block, 0, s, src, (long long)n_rows, codes, scales);
  }
  return hipGetLastError() == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

meda_status meda_dequantize_fp8(const uint8_t* codes, const float* scales, int32_t dtype, int64_t n_rows,
                                int32_t head_dim, void* rows, void* hip_stream) {
  using namespace meda;
  if (n_rows < 0) return MEDA_ERR_INVALID_ARG;
  if (dtype != MEDA_F32 && dtype != MEDA_BF16) return MEDA_ERR_UNSUPPORTED;
  if (head_dim != 64 && head_dim != 128) return MEDA_ERR_UNSUPPORTED;
  if (n_rows == 0) return MEDA_OK;
  if (!rows || !codes || !scales) return MEDA_ERR_INVALID_ARG;
  if (((uintptr_t)rows | (uintptr_t)codes) & 15u || ((uintptr_t)scales & 3u)) return MEDA_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* dst = static_cast<char*>(rows);
  const int lpr = dtype == MEDA_BF16 ? head_dim / 8 : head_dim / 4;
  const dim3 grid(stream_grid(n_rows, 64 / lpr)), block(256);
  if (dtype == MEDA_BF16) {
    if (head_dim == 128) hipLaunchKernelGGL((dequantize_fp8_kernel<bf16_t, 128>), grid, block, 0, s, codes, scales, (long long)n_rows, dst);
    else hipLaunchKernelGGL((dequantize_fp8_kernel<bf16_t, 64>), grid, block, 0, s, codes, scales, (long long)n_rows, dst);
  } else {
    if (head_dim == 128) hipLaunchKernelGGL((dequantize_fp8_kernel<float, 128>), grid, block, 0, s, codes, scales, (long long)n_rows, dst);
    else hipLaunchKernelGGL((dequantize_fp8_kernel<float, 64>), grid, block, 0, s, codes, scales, (long long)n_rows, dst);
  }
  return hipGetLastError() == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

}  // extern "C"
