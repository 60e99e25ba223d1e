// One decoding step over the ragged compressed cache: out = Softmax(q K^T / sqrt(d)) V per layer and
// query head (Section 3.1, "Decoding with Multimodal KV Cache"), the cache being the rows the
// compression pass kept for the layer (S_l per kv head, Section 3.2) followed by the rows appended
// since (K = [K, k_t], V = [V, v_t]).
//
// The step reads every cached key and value once and does 4*G*d flops per (key, value) pair, so for
// the group sizes of the workloads it is bound by HBM: the kernels are plain streaming kernels (no
// LDS staging of the cache, no matrix unit).  The rows of one (layer, kv head) are cut into NS
// equal chunks; one workgroup takes one chunk for all G query heads of the group (flash-decoding
// style: a running maximum, normaliser and weighted value sum per head), a second small kernel merges
// the chunks.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/meda.h"
#include "device_utils.hpp"
#include "fp8.hpp"

namespace meda {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecRowsPerGroup = 128;  // rows a workgroup should get at the average layer budget, per query head of the group (up to 4)
constexpr int kDecMaxSplit = 64;

struct DecodeArgs {
  const char* q;            // [L][Hq][d]
  const char* k_cache;      // ragged, layer l at row off[l]*Hkv: [Hkv][S_l][d]
  const char* v_cache;
  const int32_t* layer_len; // [L]   S_l
  const int64_t* layer_off; // [L+1]
  const char* k_new;        // [L][Hkv][n_new][d] or null
  const char* v_new;
  char* out;                // [L][Hq][d]
  float* part;              // [L][Hq][NP][d + 2]: weighted value sum, maximum (base-2 logits), normaliser
  int L, Hq, Hkv, G, n_new;
  int NS, NSN, NP;          // chunks of the cached rows, chunks of the appended rows, NS + NSN
  float scale_log2;
  // 8-bit cache (FP8 instantiation): k_cache / v_cache hold E4M3 codes, one scale per row
  const float* k_scale;     // [B*Hkv]
  const float* v_scale;
  int sp0;                  // chunk index of the launch's first workgroup (the appended rows of an 8-bit cache
                            // are taken by a second launch of the plain kernel, which starts at NS)
};

// 8-byte load of data that is read once (see load16_stream)
__device__ __forceinline__ uint2 load8_stream(const void* p) {
  typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
  const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
  return make_uint2(t.x, t.y);
}

template <typename T>
struct Elems;
template <>
struct Elems<bf16_t> {
  static constexpr int kPerPiece = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  // sum of the 8 products of two packed pieces (packed dot instruction: exact products, fp32 sums)
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, x[i]), __builtin_bit_cast(bf16x2_t, y[i]), d, false);
    return d;
  }
  static __device__ __forceinline__ void store(char* dst, float x) {
    *reinterpret_cast<uint16_t*>(dst) = (uint16_t)float_to_bf16_rne(x);
  }
};
template <>
struct Elems<float> {
  static constexpr int kPerPiece = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b) {
    float d = __uint_as_float(a.x) * __uint_as_float(b.x);
    d = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), d);
    d = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), d);
    return fmaf(__uint_as_float(a.w), __uint_as_float(b.w), d);
  }
  static __device__ __forceinline__ void store(char* dst, float x) { *reinterpret_cast<float*>(dst) = x; }
};

// Value of a partner lane whose lane-index bit X differs (X = 1, 2, 4, 8 inside a row of 16 lanes: data-parallel
// primitives, no LDS traffic; the partners of 4 and 8 are the mirrored lanes of the half row / row, which differ
// in the lower bits too; X = 16: the lane 16 away).
template <int X>
__device__ __forceinline__ float lane_partner(float v) {
  const int i = __float_as_int(v);
  if constexpr (X == 1) return __int_as_float(__builtin_amdgcn_update_dpp(i, i, 0xB1, 0xF, 0xF, true));        // quad_perm 1,0,3,2
  else if constexpr (X == 2) return __int_as_float(__builtin_amdgcn_update_dpp(i, i, 0x4E, 0xF, 0xF, true));   // quad_perm 2,3,0,1
  else if constexpr (X == 4) return __int_as_float(__builtin_amdgcn_update_dpp(i, i, 0x141, 0xF, 0xF, true));  // row_half_mirror
  else if constexpr (X == 8) return __int_as_float(__builtin_amdgcn_update_dpp(i, i, 0x140, 0xF, 0xF, true));  // row_mirror
  else return __shfl_xor(v, X, kWave);
}

// The LPR lanes that read one row each hold, for every query head of the group, a partial dot product.
// RowReduceScatter sums them over the lanes and leaves in v[0] the total of ONE head per lane (the head
// row_head() names: the upper lane-index bits choose it), at GP + log2(LPR) - 1 exchanges instead of
// GP * log2(LPR); RowAllGather is the inverse: from one value per lane for that lane's head to all GP
// values in every lane.  N: values still held, X: bit in which the partner differs.  All array indices
// are compile-time constants (the arrays live in registers).
template <int GP, int N, int X>
struct RowReduceScatter {
  static __device__ __forceinline__ void run(float (&v)[GP], int cc) {
    if constexpr (X >= 1) {
      if constexpr (N > 1) {
        const bool up = (cc & X) != 0;
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
          const float keep = up ? v[i + N / 2] : v[i], send = up ? v[i] : v[i + N / 2];
          v[i] = keep + lane_partner<X>(send);
        }
        RowReduceScatter<GP, N / 2, X / 2>::run(v, cc);
      } else {
        v[0] += lane_partner<X>(v[0]);
        RowReduceScatter<GP, 1, X / 2>::run(v, cc);
      }
    }
  }
};
template <int GP, int LPR>
__device__ __forceinline__ int row_head(int cc) {
  int h = 0, n = GP;
#pragma unroll
  for (int x = LPR / 2; x >= 1; x >>= 1) {
    if (n > 1) {
      n >>= 1;
      h += (cc & x) ? n : 0;
    }
  }
  return h;
}
// N: values held so far (w[0..N)), X: partner bit of this step; the steps run from the last halving
// distance of the reduce-scatter back up to LPR / 2.
template <int GP, int N, int X>
struct RowAllGather {
  static __device__ __forceinline__ void run(float (&w)[GP], int cc) {
    if constexpr (N < GP) {
      const bool up = (cc & X) != 0;
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const float other = lane_partner<X>(w[i]);
        w[i + N] = up ? w[i] : other;
        w[i] = up ? other : w[i];
      }
      RowAllGather<GP, 2 * N, 2 * X>::run(w, cc);
    }
  }
};
template <int GP, int LPR>
__device__ __forceinline__ void row_reduce_scatter(float (&v)[GP], int cc) {
  RowReduceScatter<GP, GP, LPR / 2>::run(v, cc);
}
template <int GP, int LPR>
__device__ __forceinline__ void row_all_gather(float mine, float (&w)[GP], int cc) {
  w[0] = mine;
  RowAllGather<GP, 1, LPR / GP>::run(w, cc);   // the last halving step of the reduce-scatter had distance LPR / GP
}

// grid (NP, Hkv, L), 256 threads.  A row is read by LPR = row bytes / 16 lanes (16 bytes each), so a
// wave takes 64 / LPR rows per step; every lane group keeps, per query head of the group, the running
// maximum, the normaliser and its piece of the weighted value sum over the rows it has seen.  GP is
// the group size rounded up to a power of two (heads past G repeat head 0 and are not stored).
// FP8: the cached rows are E4M3 codes with one scale per row (8-byte pieces, converted to packed bf16 on
// arrival, which is exact; the key's scale multiplies the logit, the value's scale the softmax weight); the
// queries stay bf16 and the launch covers the cached rows only.
template <typename T, int D, int GP, bool FP8>
__global__ void __launch_bounds__(kDecThreads, 2) decode_partial_kernel(DecodeArgs a) {
  using TL = Tile<T, D>;
  using EL = Elems<T>;
  constexpr int LPR = TL::kChunksPerRow;
  constexpr int MS = 64 / LPR;
  constexpr int E = EL::kPerPiece;
  constexpr int U = 2;  // steps whose loads are issued together
  static_assert(!FP8 || sizeof(T) == 2, "the 8-bit cache is read with bf16 queries");
  constexpr size_t kCacheRowBytes = FP8 ? (size_t)D : (size_t)TL::kRowBytes;
  constexpr int kCachePieceBytes = FP8 ? E : 16;
  __shared__ float red_o[kDecWaves][GP][D];
  __shared__ float red_m[kDecWaves][GP], red_z[kDecWaves][GP];

  const int sp = blockIdx.x + a.sp0, g = blockIdx.y, l = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sub = lane / LPR, cc = lane - sub * LPR;

  // the rows of this workgroup
  const char *kb, *vb;
  const float *ksc = nullptr, *vsc = nullptr;
  int r_beg, r_end;
  size_t row_bytes = kCacheRowBytes;
  int piece_bytes = kCachePieceBytes;
  if (FP8 || sp < a.NS) {
    const int S = a.layer_len[l];
    const int chunk = (S + a.NS - 1) / a.NS;
    r_beg = sp * chunk;
    r_end = min(S, r_beg + chunk);
    const size_t row0 = (size_t)a.layer_off[l] * a.Hkv + (size_t)g * S;
    kb = a.k_cache + row0 * kCacheRowBytes;
    vb = a.v_cache + row0 * kCacheRowBytes;
    if (FP8) {
      ksc = a.k_scale + row0;
      vsc = a.v_scale + row0;
    }
  } else {
    const int chunk = (a.n_new + a.NSN - 1) / a.NSN;
    r_beg = (sp - a.NS) * chunk;
    r_end = min(a.n_new, r_beg + chunk);
    const size_t base = ((size_t)(l * a.Hkv + g) * a.n_new) * TL::kRowBytes;
    kb = a.k_new + base;
    vb = a.v_new + base;
    row_bytes = TL::kRowBytes;
    piece_bytes = 16;
  }
  kb += cc * piece_bytes;
  vb += cc * piece_bytes;

  // this lane's piece of the G queries, kept packed
  uint4 qp[GP];
#pragma unroll
  for (int h = 0; h < GP; ++h) {
    const int hq = g * a.G + (h < a.G ? h : 0);
    qp[h] = *reinterpret_cast<const uint4*>(a.q + ((size_t)(l * a.Hq + hq)) * TL::kRowBytes + cc * 16);
  }
  // running maximum and normaliser of the ONE head this lane evaluates (row_head), weighted value sums of all
  float m1 = kNegBig, z1 = 0.f, o[GP][E];
#pragma unroll
  for (int h = 0; h < GP; ++h)
#pragma unroll
    for (int e = 0; e < E; ++e) o[h][e] = 0.f;

  for (int r0 = r_beg + wave * MS; r0 < r_end; r0 += U * kDecWaves * MS) {
    uint4 kv[U], vv[U];
    float sck[U], scv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = r0 + u * kDecWaves * MS + sub;
      ok[u] = r < r_end;
      const int rc = min(r, r_end - 1);  // rows past the end repeat the last one
      const size_t ro = (size_t)rc * row_bytes;
      if constexpr (FP8) {
        const uint2 kc = load8_stream(kb + ro), vc = load8_stream(vb + ro);
        sck[u] = ksc[rc];
        scv[u] = vsc[rc];
        kv[u] = e4m3x8_to_bf16x8(kc);          // keys as packed bf16 for the dot instruction
        vv[u] = make_uint4(vc.x, vc.y, 0u, 0u);  // values stay codes until they are needed as floats
      } else {
        kv[u] = load16_stream(kb + ro);
        vv[u] = load16_stream(vb + ro);
        sck[u] = scv[u] = 1.0f;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s[GP];
#pragma unroll
      for (int h = 0; h < GP; ++h) s[h] = EL::dot(qp[h], kv[u]);
      row_reduce_scatter<GP, LPR>(s, cc);
      const float s1 = ok[u] ? (FP8 ? s[0] * sck[u] * a.scale_log2 : s[0] * a.scale_log2) : kNegBig;
      // a new maximum of some head in some lane group: rescale what that head has so far (rare after
      // the first rows)
      if (__ballot(s1 > m1) != 0ull) {
        const float mn = fmaxf(m1, s1);
        const float c1 = __builtin_amdgcn_exp2f(m1 - mn);
        z1 *= c1;
        m1 = mn;
        float c[GP];
        row_all_gather<GP, LPR>(c1, c, cc);
#pragma unroll
        for (int h = 0; h < GP; ++h)
#pragma unroll
          for (int e = 0; e < E; ++e) o[h][e] *= c[h];
      }
      const float p1 = ok[u] ? __builtin_amdgcn_exp2f(s1 - m1) : 0.f;
      z1 += p1;
      float p[GP], vf[E];
      row_all_gather<GP, LPR>(FP8 ? p1 * scv[u] : p1, p, cc);   // the value row's scale rides on its weight
      if constexpr (FP8) {
        e4m3x2_to_float(vv[u].x, false, vf[0], vf[1]);
        e4m3x2_to_float(vv[u].x, true, vf[2], vf[3]);
        e4m3x2_to_float(vv[u].y, false, vf[4], vf[5]);
        e4m3x2_to_float(vv[u].y, true, vf[6], vf[7]);
      } else {
        EL::unpack(vv[u], vf);
      }
#pragma unroll
      for (int h = 0; h < GP; ++h)
#pragma unroll
        for (int e = 0; e < E; ++e) o[h][e] = fmaf(p[h], vf[e], o[h][e]);
    }
  }
  float m[GP], z[GP];
  row_all_gather<GP, LPR>(m1, m, cc);
  row_all_gather<GP, LPR>(z1, z, cc);

  // merge the lane groups of the wave (they saw different rows), then the waves through LDS
#pragma unroll
  for (int x = LPR; x < 64; x <<= 1) {
#pragma unroll
    for (int h = 0; h < GP; ++h) {
      const float mo = __shfl_xor(m[h], x, kWave), zo = __shfl_xor(z[h], x, kWave);
      const float mn = fmaxf(m[h], mo);
      const float c0 = __builtin_amdgcn_exp2f(m[h] - mn), c1 = __builtin_amdgcn_exp2f(mo - mn);
      z[h] = z[h] * c0 + zo * c1;
#pragma unroll
      for (int e = 0; e < E; ++e) o[h][e] = o[h][e] * c0 + __shfl_xor(o[h][e], x, kWave) * c1;
      m[h] = mn;
    }
  }
  if (sub == 0) {
#pragma unroll
    for (int h = 0; h < GP; ++h) {
#pragma unroll
      for (int e = 0; e < E; ++e) red_o[wave][h][cc * E + e] = o[h][e];
      if (cc == 0) {
        red_m[wave][h] = m[h];
        red_z[wave][h] = z[h];
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < a.G * D; i += kDecThreads) {
    const int h = i / D, j = i - h * D;
    float mn = red_m[0][h];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mn = fmaxf(mn, red_m[w][h]);
    float zs = 0.f, os = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float c = __builtin_amdgcn_exp2f(red_m[w][h] - mn);
      zs = fmaf(red_z[w][h], c, zs);
      os = fmaf(red_o[w][h][j], c, os);
    }
    float* dst = a.part + ((size_t)(l * a.Hq + g * a.G + h) * a.NP + sp) * (D + 2);
    dst[j] = os;
    if (j == 0) {
      dst[D] = mn;
      dst[D + 1] = zs;
    }
  }
}

// The same partial step on the matrix unit, for bf16 rows of 128 elements and groups of 5 to 8 query heads, where
// the kernel above is bound by the vector ALU (about 160 vector instructions per 32 bytes a lane reads) and not by
// HBM.  A wave takes 16 rows per step:
//   logits  D[key][head] = sum_d K[key][d] Q[head][d]    4 x v_mfma_f32_16x16x32_bf16 (exact products, fp32 sums)
//   output  O[head][col] += sum_key P[key][head] V[key][col]   32 x v_mfma_f32_16x16x4_f32 (fp32 weights and values)
// Lane l = (c, g) = (l % 16, l / 16).  For the logits it holds the pieces g, 4+g, 8+g, 12+g (16 bytes each) of key c
// and of query head c, and receives the logits of head c for the keys 4g .. 4g+3.  The second product runs over the
// keys in four instructions i = 0..3, instruction i taking the keys {4g' + i} with g' as its k index: its weight
// operand is then this lane's own register i (no cross-lane movement), and its value operand element j of piece c of
// key 4g + i, which the lane loads itself.  Output column 8c + j of the heads 4g .. 4g+3 accumulates in this lane.
// The running maximum of a head is kept common to the four lane groups (they hold different keys of the same
// head); the normaliser is summed per group and merged at the end.
constexpr int kDecMfmaRows = 16;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// FP8: the cached rows are E4M3 codes with one scale per row (pieces of 8 bytes; keys become packed bf16 on arrival,
// which is exact, and the key's scale multiplies the logit; values become fp32 and their scale rides on the weight);
// the launch then covers the cached rows only.
template <int D, bool FP8>
__global__ void __launch_bounds__(kDecThreads, 2) decode_partial_mfma_kernel(DecodeArgs a) {
  static_assert(D == 128, "16 pieces per row: one per lane of a lane group");
  constexpr int kRowBytes = D * 2;                     // bf16 rows (queries, appended rows, the bf16 cache)
  constexpr int kCacheRowBytes = FP8 ? D : kRowBytes;  // rows of the cache this launch reads
  constexpr int kPiece = FP8 ? 8 : 16;
  constexpr int GPM = 16;  // heads the matrix shapes hold (a.G <= 8 of them are real)
  __shared__ float red_o[kDecWaves][8][D];
  __shared__ float red_m[kDecWaves][8], red_z[kDecWaves][8];

  const int sp = blockIdx.x + a.sp0, g = blockIdx.y, l = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, grp = lane >> 4;

  const char *kb, *vb;
  const float *ksc = nullptr, *vsc = nullptr;
  int r_beg, r_end;
  if (FP8 || sp < a.NS) {
    const int S = a.layer_len[l];
    const int chunk = (S + a.NS - 1) / a.NS;
    r_beg = sp * chunk;
    r_end = min(S, r_beg + chunk);
    const size_t row0 = (size_t)a.layer_off[l] * a.Hkv + (size_t)g * S;
    kb = a.k_cache + row0 * kCacheRowBytes;
    vb = a.v_cache + row0 * kCacheRowBytes;
    if (FP8) {
      ksc = a.k_scale + row0;
      vsc = a.v_scale + row0;
    }
  } else {
    const int chunk = (a.n_new + a.NSN - 1) / a.NSN;
    r_beg = (sp - a.NS) * chunk;
    r_end = min(a.n_new, r_beg + chunk);
    const size_t base = ((size_t)(l * a.Hkv + g) * a.n_new) * kRowBytes;
    kb = a.k_new + base;
    vb = a.v_new + base;
  }

  // query head c of the group (heads past G: zeros, their columns are dropped)
  uint4 qp[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qp[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (c < a.G) qp[ks] = *reinterpret_cast<const uint4*>(a.q + (size_t)(l * a.Hq + g * a.G + c) * kRowBytes + (4 * ks + grp) * 16);
  }

  float m_run = kNegBig, z_run = 0.f;  // of head c; m_run is the same in the four lane groups
  f32x4_t acc[8];                      // acc[j][r]: output column 8c + j of head 4 grp + r
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // a step's loads: four key pieces (packed bf16 after the load), four value pieces (codes stay codes until they
  // are needed as floats), and with FP8 the scales of the keys 4 grp + i this lane has logits and weights for
  auto load_step = [&](int r0, uint4 (&kv)[4], uint4 (&vv)[4], float (&sk)[4], float (&sv)[4]) {
    const int rk = min(r0 + c, r_end - 1);  // rows past the end repeat the last one (their weights are zero)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const char* src = kb + (size_t)rk * kCacheRowBytes + (4 * ks + grp) * kPiece;
      if constexpr (FP8) kv[ks] = e4m3x8_to_bf16x8(load8_stream(src)); else kv[ks] = load16_stream(src);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rv = min(r0 + 4 * grp + i, r_end - 1);
      const char* src = vb + (size_t)rv * kCacheRowBytes + c * kPiece;
      if constexpr (FP8) {
        const uint2 vc = load8_stream(src);
        vv[i] = make_uint4(vc.x, vc.y, 0u, 0u);
        sk[i] = ksc[rv];
        sv[i] = vsc[rv];
      } else {
        vv[i] = load16_stream(src);
        sk[i] = sv[i] = 1.0f;
      }
    }
  };

  constexpr int kStepStride = kDecWaves * kDecMfmaRows;
  int r0 = r_beg + wave * kDecMfmaRows;
  uint4 kv[4], vv[4];
  float sk[4], sv[4];
  if (r0 < r_end) load_step(r0, kv, vv, sk, sv);
  for (; r0 < r_end; r0 += kStepStride) {
    uint4 kn[4], vn[4];
    float skn[4], svn[4];
    const bool more = r0 + kStepStride < r_end;
    if (more) load_step(r0 + kStepStride, kn, vn, skn, svn);  // in flight while this step is computed

    f32x4_t s4 = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv[ks]), __builtin_bit_cast(bf16x8_t, qp[ks]),
                                                   s4, 0, 0, 0);
    // this lane: head c, keys r0 + 4 grp + i
    float t[4];
    float bm = kNegBig;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      t[i] = (r0 + 4 * grp + i < r_end) ? (FP8 ? s4[i] * sk[i] * a.scale_log2 : s4[i] * a.scale_log2) : kNegBig;
      bm = fmaxf(bm, t[i]);
    }
    bm = fmaxf(bm, __shfl_xor(bm, 16, kWave));
    bm = fmaxf(bm, __shfl_xor(bm, 32, kWave));
    if (__ballot(bm > m_run) != 0ull) {  // a new maximum of some head: rescale what that head has so far (rare)
      const float mn = fmaxf(m_run, bm);
      const float c1 = __builtin_amdgcn_exp2f(m_run - mn);
      z_run *= c1;
      m_run = mn;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float cr = __shfl(c1, 4 * grp + r, kWave);  // the factor of head 4 grp + r (lane 4 grp + r of group 0)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j][r] *= cr;
      }
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = (r0 + 4 * grp + i < r_end) ? __builtin_amdgcn_exp2f(t[i] - m_run) : 0.f;
      z_run += p[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float vf[8];
      if constexpr (FP8) {
        e4m3x2_to_float(vv[i].x, false, vf[0], vf[1]);
        e4m3x2_to_float(vv[i].x, true, vf[2], vf[3]);
        e4m3x2_to_float(vv[i].y, false, vf[4], vf[5]);
        e4m3x2_to_float(vv[i].y, true, vf[6], vf[7]);
      } else {
        Elems<bf16_t>::unpack(vv[i], vf);
      }
      const float w = FP8 ? p[i] * sv[i] : p[i];  // the value row's scale rides on its weight
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(w, vf[j], acc[j], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kv[i] = kn[i];
        vv[i] = vn[i];
        sk[i] = skn[i];
        sv[i] = svn[i];
      }
    }
  }
  // the four lane groups saw different keys of head c: one normaliser
  z_run += __shfl_xor(z_run, 16, kWave);
  z_run += __shfl_xor(z_run, 32, kWave);

  // merge the waves through LDS (as in the kernel above)
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int h = 4 * grp + r;
    if (h < 8) {
#pragma unroll
      for (int j = 0; j < 8; ++j) red_o[wave][h][8 * c + j] = acc[j][r];
    }
  }
  if (grp == 0 && c < 8) {
    red_m[wave][c] = m_run;
    red_z[wave][c] = z_run;
  }
  __syncthreads();
  for (int i = tid; i < a.G * D; i += kDecThreads) {
    const int h = i / D, j = i - h * D;
    float mn = red_m[0][h];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mn = fmaxf(mn, red_m[w][h]);
    float zs = 0.f, os = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float cw = __builtin_amdgcn_exp2f(red_m[w][h] - mn);
      zs = fmaf(red_z[w][h], cw, zs);
      os = fmaf(red_o[w][h][j], cw, os);
    }
    float* dst = a.part + ((size_t)(l * a.Hq + g * a.G + h) * a.NP + sp) * (D + 2);
    dst[j] = os;
    if (j == 0) {
      dst[D] = mn;
      dst[D + 1] = zs;
    }
  }
}

// grid (Hq, L), D threads: merges the NP chunks of one query head and writes the output row.
template <typename T, int D>
__global__ void __launch_bounds__(D) decode_combine_kernel(DecodeArgs a) {
  const int h = blockIdx.x, l = blockIdx.y, j = threadIdx.x;
  const float* p = a.part + (size_t)(l * a.Hq + h) * a.NP * (D + 2);
  float mn = kNegBig;
  for (int s = 0; s < a.NP; ++s) mn = fmaxf(mn, p[(size_t)s * (D + 2) + D]);
  float zs = 0.f, os = 0.f;
  for (int s = 0; s < a.NP; ++s) {
    const float* ps = p + (size_t)s * (D + 2);
    const float c = __builtin_amdgcn_exp2f(ps[D] - mn);
    zs = fmaf(ps[D + 1], c, zs);
    os = fmaf(ps[j], c, os);
  }
  Elems<T>::store(a.out + ((size_t)(l * a.Hq + h) * D + j) * sizeof(T), os / zs);
}

struct DecodePlan {
  int L, Hq, Hkv, G, GP, d, dtype, n_new, NS, NSN, NP;
  float scale_log2;
  size_t ws_bytes;
};

static meda_status make_decode_plan(const meda_decode_params* p, DecodePlan* pl) {
  if (!p) return MEDA_ERR_INVALID_ARG;
  if (p->n_layers < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_new < 0) return MEDA_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return MEDA_ERR_INVALID_ARG;
  if (p->total_budget < p->n_layers) return MEDA_ERR_BUDGET;  // every layer keeps at least one row
  if (!(p->softmax_scale >= 0.0f) || !isfinite(p->softmax_scale)) return MEDA_ERR_INVALID_ARG;
  if (p->dtype != MEDA_F32 && p->dtype != MEDA_BF16) return MEDA_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return MEDA_ERR_UNSUPPORTED;
  const int G = p->n_q_heads / p->n_kv_heads;
  if (G > 8 || p->n_layers > 65535 || p->n_kv_heads > 65535) return MEDA_ERR_UNSUPPORTED;
  if ((int64_t)p->n_layers * p->n_q_heads >= (1ll << 24)) return MEDA_ERR_UNSUPPORTED;  // (layer, head) ids are ints
  pl->L = p->n_layers; pl->Hq = p->n_q_heads; pl->Hkv = p->n_kv_heads; pl->G = G; pl->d = p->head_dim;
  pl->GP = G <= 1 ? 1 : (G <= 2 ? 2 : (G <= 4 ? 4 : 8));
  pl->dtype = p->dtype; pl->n_new = p->n_new;
  // the per-head state a workgroup merges at its end grows with the group size: give it more rows then
  const int rows_per_group = kDecRowsPerGroup * (pl->GP < 4 ? pl->GP : 4);
  const int64_t avg = p->total_budget / p->n_layers;
  int64_t ns = (avg + rows_per_group - 1) / rows_per_group;
  pl->NS = (int)(ns < 1 ? 1 : (ns > kDecMaxSplit ? kDecMaxSplit : ns));
  int64_t nsn = ((int64_t)p->n_new + kDecRowsPerGroup - 1) / kDecRowsPerGroup;
  pl->NSN = (int)(nsn > kDecMaxSplit ? kDecMaxSplit : nsn);
  pl->NP = pl->NS + pl->NSN;
  const double scale = p->softmax_scale > 0.0f ? (double)p->softmax_scale : 1.0 / sqrt((double)p->head_dim);
  pl->scale_log2 = (float)(scale * 1.4426950408889634074);
  pl->ws_bytes = ((size_t)pl->L * pl->Hq * pl->NP * (pl->d + 2) * sizeof(float) + 255) / 256 * 256;
  return MEDA_OK;
}

template <typename T, int D, int GP>
static hipError_t launch_decode_g(const DecodePlan& pl, const DecodeArgs& a_in, hipStream_t s) {
  DecodeArgs a = a_in;
  hipError_t e;
  if constexpr (sizeof(T) == 2) {
    if (a.k_scale) {  // 8-bit cache: its rows first, then the appended bf16 rows with the plain kernel
      constexpr bool kMfma = D == 128 && GP == 8;  // groups of 5 to 8 heads: the matrix form (see its comment)
      a.sp0 = 0;
      if constexpr (kMfma)
        hipLaunchKernelGGL((decode_partial_mfma_kernel<D, true>), dim3(pl.NS, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
      else
        hipLaunchKernelGGL((decode_partial_kernel<T, D, GP, true>), dim3(pl.NS, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
      if (pl.NSN > 0) {
        a.sp0 = pl.NS;
        if constexpr (kMfma)
          hipLaunchKernelGGL((decode_partial_mfma_kernel<D, false>), dim3(pl.NSN, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
        else
          hipLaunchKernelGGL((decode_partial_kernel<T, D, GP, false>), dim3(pl.NSN, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
      hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(pl.Hq, pl.L), dim3(D), 0, s, a);
      return hipGetLastError();
    }
  }
  a.sp0 = 0;
  if constexpr (sizeof(T) == 2 && D == 128 && GP == 8) {
    // groups of 5 to 8 heads: the vector form is bound by its instruction count, the matrix form by HBM
    hipLaunchKernelGGL((decode_partial_mfma_kernel<D, false>), dim3(pl.NP, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
  } else {
    hipLaunchKernelGGL((decode_partial_kernel<T, D, GP, false>), dim3(pl.NP, pl.Hkv, pl.L), dim3(kDecThreads), 0, s, a);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(pl.Hq, pl.L), dim3(D), 0, s, a);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_decode_t(const DecodePlan& pl, const DecodeArgs& a, hipStream_t s) {
  switch (pl.GP) {
    case 1: return launch_decode_g<T, D, 1>(pl, a, s);
    case 2: return launch_decode_g<T, D, 2>(pl, a, s);
    case 4: return launch_decode_g<T, D, 4>(pl, a, s);
    default: return launch_decode_g<T, D, 8>(pl, a, s);
  }
}

// Scratch of the entry point that allocates nothing: the chunk partials of one decoding step live in this
// file-scope device array instead of a caller-provided workspace.  Every GPU holds its own copy at its own
// address; the name below is only the host-side handle of the symbol, the address a kernel can use is looked
// up once per device (scratch_of_current_device) and kept.
constexpr size_t kDecodeScratchBytes = (size_t)MEDA_DECODE_NOALLOC_MAX_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kDecodeScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device, or null (with *err set) if a HIP call failed.
static void* scratch_of_current_device(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !ptr) {
      if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace meda

extern "C" {

size_t meda_decode_workspace_bytes(const meda_decode_params* params) {
  meda::DecodePlan pl;
  return meda::make_decode_plan(params, &pl) == MEDA_OK ? pl.ws_bytes : 0;
}

static meda_status decode_common(const meda_decode_params* params, const void* q, const void* k_cache,
                                 const void* v_cache, const float* k_scale, const float* v_scale, bool fp8,
                                 const int32_t* layer_len, const int64_t* layer_off, const void* k_new,
                                 const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  using namespace meda;
  DecodePlan pl;
  const meda_status st = make_decode_plan(params, &pl);
  if (st != MEDA_OK) return st;
  if (fp8 && pl.dtype != MEDA_BF16) return MEDA_ERR_UNSUPPORTED;
  if (!q || !k_cache || !v_cache || !layer_len || !layer_off || !out) return MEDA_ERR_INVALID_ARG;
  if (fp8 && (!k_scale || !v_scale || (((uintptr_t)k_scale | (uintptr_t)v_scale) & 3u))) return MEDA_ERR_INVALID_ARG;
  if (pl.n_new > 0 && (!k_new || !v_new)) return MEDA_ERR_INVALID_ARG;
  const uintptr_t al = (uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)k_new | (uintptr_t)v_new;
  if (al & 15u) return MEDA_ERR_INVALID_ARG;  // rows are moved in 16-byte pieces
  if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < pl.ws_bytes) return MEDA_ERR_WORKSPACE;

  DecodeArgs a;
  a.q = static_cast<const char*>(q);
  a.k_cache = static_cast<const char*>(k_cache);
  a.v_cache = static_cast<const char*>(v_cache);
  a.layer_len = layer_len;
  a.layer_off = layer_off;
  a.k_new = static_cast<const char*>(k_new);
  a.v_new = static_cast<const char*>(v_new);
  a.out = static_cast<char*>(out);
  a.part = static_cast<float*>(workspace);
  a.L = pl.L; a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.n_new = pl.n_new;
  a.NS = pl.NS; a.NSN = pl.NSN; a.NP = pl.NP;
  a.scale_log2 = pl.scale_log2;
  a.k_scale = fp8 ? k_scale : nullptr;
  a.v_scale = fp8 ? v_scale : nullptr;
  a.sp0 = 0;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (pl.dtype == MEDA_BF16) e = pl.d == 128 ? launch_decode_t<bf16_t, 128>(pl, a, s) : launch_decode_t<bf16_t, 64>(pl, a, s);
  else e = pl.d == 128 ? launch_decode_t<float, 128>(pl, a, s) : launch_decode_t<float, 64>(pl, a, s);
  return e == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

meda_status meda_decode_attention(const meda_decode_params* params, const void* q, const void* k_cache,
                                  const void* v_cache, const int32_t* layer_len, const int64_t* layer_off,
                                  const void* k_new, const void* v_new, void* out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  return decode_common(params, q, k_cache, v_cache, nullptr, nullptr, false, layer_len, layer_off, k_new, v_new, out,
                       workspace, workspace_bytes, hip_stream);
}

meda_status meda_decode_attention_noalloc(const meda_decode_params* params, const void* q, const void* k_cache,
                                          const void* v_cache, const int32_t* layer_len, const int64_t* layer_off,
                                          const void* k_new, const void* v_new, void* out, void* hip_stream) {
  meda::DecodePlan pl;
  const meda_status st = meda::make_decode_plan(params, &pl);
  if (st != MEDA_OK) return st;
  if (pl.ws_bytes > meda::kDecodeScratchBytes) return MEDA_ERR_SCRATCH_LIMIT;
  hipError_t err = hipSuccess;
  void* ptr = meda::scratch_of_current_device(&err);
  if (!ptr) return MEDA_ERR_HIP;
  // every chunk partial the combine kernel reads is written by the partial kernel of the same call (also for
  // chunks without rows), so nothing in the array has to be cleared between calls
  return decode_common(params, q, k_cache, v_cache, nullptr, nullptr, false, layer_len, layer_off, k_new, v_new, out,
                       ptr, meda::kDecodeScratchBytes, hip_stream);
}

meda_status meda_decode_attention_fp8(const meda_decode_params* params, const void* q, const uint8_t* k_codes,
                                      const uint8_t* v_codes, const float* k_scales, const float* v_scales,
                                      const int32_t* layer_len, const int64_t* layer_off, const void* k_new,
                                      const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
  return decode_common(params, q, k_codes, v_codes, k_scales, v_scales, true, layer_len, layer_off, k_new, v_new, out,
                       workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
