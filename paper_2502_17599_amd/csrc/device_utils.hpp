// Device-side building blocks shared by the kernels: MFMA fragments for "row times row" products
// (both operands stored with the head dimension contiguous), padded LDS tiles, rounding.
//
// Fragment convention.  A 32x32 MFMA block multiplies 32 rows of operand A by 32 rows of operand B
// over the whole head dimension.  Lane l holds, for row (l % 32), the half of the row selected by
// (l / 32): elements [ (l/32)*D/2, (l/32+1)*D/2 ).  The MFMA pairs element e of A's lane group with
// element e of B's lane group, so any assignment of row elements to (lane group, step) gives the
// same dot product as long as both operands use the same one; taking contiguous halves lets every
// lane fetch its fragment with 16-byte loads from one contiguous run.
// Result layout of a 32x32 block (f32x16 acc): acc[r] is the product of A row
// (r/4)*8 + (l/32)*4 + (r%4) with B row (l % 32).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace meda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

struct bf16_t {
  uint16_t bits;
};

constexpr int kWave = 64;
constexpr float kNegBig = -1.0e30f;

template <typename T, int D>
struct Tile {
  static constexpr int kRowBytes = D * (int)sizeof(T);
  static constexpr int kStride = kRowBytes + 16;  // LDS row stride: the 16-byte pad spreads 16-byte reads of
                                                  // consecutive rows over all banks
  static constexpr int kChunksPerRow = kRowBytes / 16;
  static constexpr int kFragChunks = kRowBytes / 32;  // 16-byte chunks a lane holds per fragment
  static constexpr int kHalfBytes = kRowBytes / 2;
};

template <typename T, int D>
struct Frag {
  uint4 c[Tile<T, D>::kFragChunks];
};

// Row of the A operand that accumulator register r of this lane belongs to.
__device__ __forceinline__ int acc_row(int r, int lane_group) { return (r >> 2) * 8 + lane_group * 4 + (r & 3); }

template <typename T, int D>
__device__ __forceinline__ void frag_zero(Frag<T, D>& f) {
#pragma unroll
  for (int i = 0; i < Tile<T, D>::kFragChunks; ++i) f.c[i] = make_uint4(0, 0, 0, 0);
}

// Fragment of one row stored contiguously at `row_ptr` (global or LDS).
template <typename T, int D>
__device__ __forceinline__ void frag_load(Frag<T, D>& f, const char* row_ptr, int lane_group) {
  const uint4* p = reinterpret_cast<const uint4*>(row_ptr + lane_group * Tile<T, D>::kHalfBytes);
#pragma unroll
  for (int i = 0; i < Tile<T, D>::kFragChunks; ++i) f.c[i] = p[i];
}

template <typename T, int D>
__device__ __forceinline__ void mma(f32x16_t& acc, const Frag<T, D>& a, const Frag<T, D>& b);

template <>
__device__ __forceinline__ void mma<bf16_t, 128>(f32x16_t& acc, const Frag<bf16_t, 128>& a,
                                                 const Frag<bf16_t, 128>& b) {
#pragma unroll
  for (int i = 0; i < Tile<bf16_t, 128>::kFragChunks; ++i)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a.c[i]),
                                                  __builtin_bit_cast(bf16x8_t, b.c[i]), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma<bf16_t, 64>(f32x16_t& acc, const Frag<bf16_t, 64>& a,
                                                const Frag<bf16_t, 64>& b) {
#pragma unroll
  for (int i = 0; i < Tile<bf16_t, 64>::kFragChunks; ++i)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a.c[i]),
                                                  __builtin_bit_cast(bf16x8_t, b.c[i]), acc, 0, 0, 0);
}

__device__ __forceinline__ void mma_f32_chunk(f32x16_t& acc, const uint4& a, const uint4& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma<float, 64>(f32x16_t& acc, const Frag<float, 64>& a,
                                               const Frag<float, 64>& b) {
#pragma unroll
  for (int i = 0; i < Tile<float, 64>::kFragChunks; ++i) mma_f32_chunk(acc, a.c[i], b.c[i]);
}
template <>
__device__ __forceinline__ void mma<float, 128>(f32x16_t& acc, const Frag<float, 128>& a,
                                                const Frag<float, 128>& b) {
#pragma unroll
  for (int i = 0; i < Tile<float, 128>::kFragChunks; ++i) mma_f32_chunk(acc, a.c[i], b.c[i]);
}

__device__ __forceinline__ f32x16_t acc_zero() {
  f32x16_t z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.0f;
  return z;
}

// 16-byte load of data that is read once and not again soon: the non-temporal hint keeps such a stream
// from displacing reusable lines in the caches, and streams measurably faster from HBM.
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// 16-byte store of data this kernel does not read again (same hint as load16_stream).
__device__ __forceinline__ void store16_stream(void* p, const uint4& v) {
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
}

// 16 (or 4) bytes per lane from global memory straight into LDS, without passing through registers: lane i's
// piece, read at gbase + goff (gbase the same for every lane of the wave, goff this lane's byte offset),
// lands at LDS byte address lds_base + 16 i (4 i), lds_base being the same for every lane.  The copy is
// asynchronous and counted like a global load; the compiler does not know that it writes LDS, so the wave that
// issued copies waits for them itself with async_copy_wait<N>() (returns when at most N of its copies, the
// youngest ones, are still in flight) and a barrier after that wait publishes them to the other waves.
__device__ __forceinline__ void async_copy16_to_lds(const void* gbase, unsigned goff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(goff), "s"(gbase), "s"(lds_base) : "memory");
}
// A pointer that is the same in every lane, as a value the compiler knows to be uniform (64-bit address arithmetic
// is done on the vector unit, and the copies above need their base in scalar registers).
template <typename P>
__device__ __forceinline__ const P* uniform_ptr(const P* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const P*>(((unsigned long long)hi << 32) | lo);
}
// The same copy with the non-temporal hint: for data that is read once (a stream) and should not push data that
// other workgroups are about to re-read out of the L2.
__device__ __forceinline__ void async_copy16_to_lds_stream(const void* gbase, unsigned goff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(goff), "s"(gbase), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void async_copy4_to_lds(const void* gbase, unsigned goff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(goff), "s"(gbase), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void async_copy_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Tiles filled by these copies cannot pad their rows (a copy instruction writes lane i's 16 bytes at base + 16 i), so
// the 16-byte chunk c of row r is kept at position c ^ swizzle_of_row(r) of the row: which global chunk a lane
// fetches is free, and the xor spreads the 16 rows a fragment load touches in one pass over all banks (rows of 256
// bytes or more start at the same bank: r mod 16; two rows of 128 bytes share a bank line: (r / 2) mod 8).
template <typename T, int D>
__device__ __forceinline__ int swizzle_of_row(int r) {
  return Tile<T, D>::kRowBytes >= 256 ? (r & 15) : ((r >> 1) & 7);
}

// Copy `rows` consecutive rows (contiguous in global memory) into a padded LDS tile; rows at or
// beyond `rows_valid` are zero-filled.
template <typename T, int D>
__device__ __forceinline__ void tile_load_contiguous(char* lds, const char* gsrc, int rows, int rows_valid,
                                                     int tid, int n_threads) {
  constexpr int CPR = Tile<T, D>::kChunksPerRow;
  const int total = rows * CPR;
  for (int c = tid; c < total; c += n_threads) {
    const int row = c / CPR, cc = c - row * CPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rows_valid) v = *reinterpret_cast<const uint4*>(gsrc + (size_t)row * Tile<T, D>::kRowBytes + cc * 16);
    *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kStride + cc * 16) = v;
  }
}

// A tile of ROWS consecutive rows, cut in 16-byte pieces that are dealt round-robin to the threads of
// the workgroup and held in registers between the global loads (all issued back to back, so they are
// in flight together) and the stores into the padded LDS tile.  PIECES is sized for NTHR threads;
// larger workgroups leave the upper pieces unused.
template <typename T, int D, int ROWS, int NTHR = 256>
struct TileStage {
  static constexpr int CPR = Tile<T, D>::kChunksPerRow;
  static constexpr int TOTAL = ROWS * CPR;
  static constexpr int PIECES = (TOTAL + NTHR - 1) / NTHR;
  uint4 r[PIECES];

  // STREAM: the tile is not read again soon (a pass over the key cache), see load16_stream
  template <bool STREAM = false>
  __device__ __forceinline__ void fetch(const char* gsrc, int rows_valid, int tid, int n_threads) {
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int c = tid + i * n_threads;
      const int row = c / CPR, cc = c - row * CPR;
      r[i] = make_uint4(0, 0, 0, 0);
      if (c < TOTAL && row < rows_valid) {
        const char* src = gsrc + (size_t)row * Tile<T, D>::kRowBytes + cc * 16;
        r[i] = STREAM ? load16_stream(src) : *reinterpret_cast<const uint4*>(src);
      }
    }
  }
  __device__ __forceinline__ void commit(char* lds, int tid, int n_threads) const {
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
      const int c = tid + i * n_threads;
      const int row = c / CPR, cc = c - row * CPR;
      if (c < TOTAL) *reinterpret_cast<uint4*>(lds + row * Tile<T, D>::kStride + cc * 16) = r[i];
    }
  }
};

// ---- element conversion -----------------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Sum of squares of the 8 bf16 (or 4 f32) elements packed in one 16-byte chunk.
template <typename T>
__device__ __forceinline__ float chunk_sumsq(const uint4& v);
template <>
__device__ __forceinline__ float chunk_sumsq<bf16_t>(const uint4& v) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  float s = 0.f;
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {  // one packed dot product per pair of elements
    const bf16x2_t p = __builtin_bit_cast(bf16x2_t, w[i]);
    s = __builtin_amdgcn_fdot2_f32_bf16(p, p, s, false);
  }
  return s;
}
template <>
__device__ __forceinline__ float chunk_sumsq<float>(const uint4& v) {
  const float a = __uint_as_float(v.x), b = __uint_as_float(v.y), c = __uint_as_float(v.z),
              d = __uint_as_float(v.w);
  return fmaf(a, a, fmaf(b, b, fmaf(c, c, d * d)));
}

// double -> float, rounding to odd (truncate, then set the last bit if anything was lost).  A value
// rounded to odd at 24 bits rounds to the same bf16 (8 bits) as the original double would.  Built on
// the hardware's nearest-even conversion: if that was inexact and went away from zero, step the bit
// pattern back by one (sign-magnitude, so the same for both signs) before setting the last bit.
__device__ __forceinline__ float double_to_float_round_odd(double x) {
  const float f = (float)x;
  const double back = (double)f;
  uint32_t u = __float_as_uint(f);
  if (back != x) u = (u - (fabs(back) > fabs(x) ? 1u : 0u)) | 1u;
  return __uint_as_float(u);
}

__device__ __forceinline__ uint32_t float_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t double_to_bf16_bits(double x) {
  return float_to_bf16_rne(double_to_float_round_odd(x));
}

// ---- wave helpers ----------------------------------------------------------------------------------

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

}  // namespace meda
