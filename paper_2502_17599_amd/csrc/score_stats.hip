// Pass A of the scoring (Sections 3.2 and 3.3): row maxima and softmax normalisers of every scoring row, and
// 1/|k| of every key; then the merge of the per-chunk partials.  The layout of the pass is described in
// score_common.hpp.
#include "score_common.hpp"

namespace meda {

// ------------------------------------------------------------------------------------------ pass A
// grid (NCH, Hkv, L), or (1, Hkv * row blocks, L) in the row-block mode (more than 128 scoring rows); NCG*CS waves.
// Wave (cg, cs) keeps NQ query fragments ((head of the group, row
// block) pairs cg*NQ .. cg*NQ+NQ-1) in registers and visits the 32-key blocks sb = cs, cs+CS, ... of
// every tile of its chunk.  The product is taken with the keys as operand A and the queries as
// operand B, so a lane owns one query row and 16 keys per block: the running (max, Z_vision, Z_text)
// of the row live in three registers per fragment and need no cross-lane traffic until the end.
//
// Two ways of bringing the key tiles into LDS.  Through registers (DMA false): the next tile is fetched into registers
// while the current one is processed, and written to a padded LDS tile between two barriers.  By asynchronous
// global-to-LDS copies (DMA true, rows of at most 256 bytes): two unpadded, xor-swizzled tiles (swizzle_of_row in
// device_utils.hpp); the copies of tile t+1 are issued when tile t starts, one wait and one barrier per tile, no
// staging registers; the modality bits of a tile's keys are ballots of two bytes per lane that every wave loads for
// itself one tile ahead.  The arithmetic is the same instruction for instruction, so the results are bit-identical.
template <typename T, int D, int NQ, int NW, bool BLOCKS, bool DMA>
__global__ void __launch_bounds__(NW * 64, (NQ == 1 && NW == 4 && sizeof(T) == 2) ? 3 : 2) score_stats_kernel(ScoreArgs a) {
  using TL = Tile<T, D>;
  constexpr int RBt = TL::kRowBytes;
  constexpr int CPR = TL::kChunksPerRow;
  constexpr int NC = TL::kFragChunks;
  constexpr int kTileBytes = kScoreTile * RBt;
  extern __shared__ __align__(16) char smem[];
  char* ktile = smem;
  uint8_t* lmask = reinterpret_cast<uint8_t*>(smem + kScoreTile * TL::kStride);  // (DMA false)

  const int ch = blockIdx.x, l = blockIdx.z;
  int g = blockIdx.y, bi = 0;
  if (BLOCKS) {  // row-block mode: this workgroup's row block (the largest blocks are dispatched first)
    bi = blockIdx.y / a.Hkv;
    g = blockIdx.y - bi * a.Hkv;
    select_row_block(a, bi);
  }
  constexpr int nthr = NW * 64;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: what derives from it stays in scalar registers
  const int lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int cgi = wave % a.NCG, cs = wave / a.NCG;
  const bool active = cs < a.CS;  // the workgroup is padded to 4 or 8 waves; spare waves only move data
  const int n_combos = a.G * a.RB;

  Frag<T, D> qf[NQ];
  float m[NQ], zv[NQ], zt[NQ];
  int qrow[NQ], qhead[NQ];
  int qlast[NQ];  // position of the last row of the fragment's 32-row block (uniform over the wave)
  int nvalid = 0;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int cidx = cgi * NQ + q;
    m[q] = kNegBig;
    zv[q] = 0.f;
    zt[q] = 0.f;
    qrow[q] = 0;
    qhead[q] = 0;
    qlast[q] = -1;
    frag_zero(qf[q]);
    if (active && cidx < n_combos) {
      nvalid = q + 1;
      const int hg = cidx / a.RB, rb = cidx - hg * a.RB;
      qhead[q] = g * a.G + hg;
      qrow[q] = rb * 32 + n;
      qlast[q] = a.T - a.W + rb * 32 + 31;
      if (qrow[q] < a.W)
        frag_load(qf[q], a.q + ((size_t)(l * a.Hq + qhead[q]) * a.q_rows + a.q_row0 + qrow[q]) * TL::kRowBytes, kg);
    }
  }

  int wave_last = -1;
#pragma unroll
  for (int q = 0; q < NQ; ++q) wave_last = max(wave_last, qlast[q]);

  const uint8_t* mask = a.mask + (size_t)(l / a.Lseq) * a.Tk;  // this layer's sequence
  const int jbeg = ch * a.CH;
  const int jend = min(a.T, jbeg + a.CH);
  const char* kbase = a.k + (size_t)(l * a.Hkv + g) * a.Tk * TL::kRowBytes;
  float* invn_out = a.inv_norm + (size_t)(l * a.Hkv + g) * a.Tk;

  TileStage<T, D, DMA ? 1 : kScoreTile, nthr> stage;
  uint8_t mreg = 0;
  // DMA: copy instruction c of this wave fills the rows (wave * PF + c) * RPI .. + RPI-1 of a tile, this lane brings
  // one 16-byte chunk; rows past the end of the sequence repeat the last key (their columns are masked below)
  constexpr int RPI = 64 / CPR;
  constexpr int PF = DMA ? kScoreTile / RPI / NW : 1;
  static_assert(!DMA || (64 % CPR == 0 && kScoreTile % (RPI * NW) == 0), "the copy instructions must tile a tile evenly");
  unsigned crow[PF], cchunk[PF], coff[NC];
  uint8_t mk0 = 0, mk1 = 0;            // modality bytes of the keys lane and 64 + lane of the next tile
  unsigned long long cur0 = 0, cur1 = 0;  // modality bits of the current tile's keys 0..63 and 64..127
  const unsigned lds0 = (unsigned)(size_t)smem;
  const char* kbase_u = uniform_ptr(kbase);
  auto issue = [&](int jt, int slot) {
#pragma unroll
    for (int c = 0; c < PF; ++c)
      async_copy16_to_lds_stream(kbase_u, (unsigned)min(jt + (int)crow[c], a.T - 1) * RBt + cchunk[c],
                                 lds0 + (unsigned)(slot * kTileBytes + (wave * PF + c) * 1024));
    mk0 = (jt + lane < a.T) ? mask[jt + lane] : 0;
    mk1 = (jt + 64 + lane < a.T) ? mask[jt + 64 + lane] : 0;
  };
  if (DMA) {
#pragma unroll
    for (int c = 0; c < PF; ++c) {
      crow[c] = (unsigned)((wave * PF + c) * RPI + lane / CPR);
      cchunk[c] = (unsigned)(((lane % CPR) ^ swizzle_of_row<T, D>((int)crow[c])) * 16);
    }
    // chunk c of this lane's fragment (chunk kg * NC + c of row n of a 32-row block)
#pragma unroll
    for (int c = 0; c < NC; ++c) coff[c] = (unsigned)(n * RBt + (((kg * NC + c) ^ swizzle_of_row<T, D>(n)) * 16));
    if (jbeg < jend) issue(jbeg, 0);
  } else if (jbeg < jend) {
    stage.template fetch<true>(kbase + (size_t)jbeg * TL::kRowBytes, min(kScoreTile, a.T - jbeg), tid, nthr);
    if (tid < kScoreTile) mreg = (jbeg + tid < a.T) ? mask[jbeg + tid] : 0;
  }
  int slot = 0;
  for (int j0 = jbeg; j0 < jend; j0 += kScoreTile, slot ^= 1) {
    const int rows_valid = min(kScoreTile, a.T - j0);
    if (DMA) {
      async_copy_wait<0>();  // this wave's pieces of the tile have landed
      __syncthreads();       // every wave's have; and nobody reads the other tile (the previous one) any more
      cur0 = __ballot(mk0 != 0);
      cur1 = __ballot(mk1 != 0);
      if (j0 + kScoreTile < jend) issue(j0 + kScoreTile, slot ^ 1);
      ktile = smem + slot * kTileBytes;
    } else {
      __syncthreads();  // the previous tile is no longer read
      stage.commit(ktile, tid, nthr);
      if (tid < kScoreTile) lmask[tid] = mreg;
      __syncthreads();
      if (j0 + kScoreTile < jend) {  // next tile's loads are in flight while this one is processed
        const int jn = j0 + kScoreTile;
        stage.template fetch<true>(kbase + (size_t)jn * TL::kRowBytes, min(kScoreTile, a.T - jn), tid, nthr);
        if (tid < kScoreTile) mreg = (jn + tid < a.T) ? mask[jn + tid] : 0;
      }
    }

    // 1/|k| of the tile's keys: two threads per row (the first row block sees every key; the others skip this)
    for (int row = tid >> 1; bi == 0 && row < kScoreTile; row += nthr >> 1) {
      float ss = 0.f;
      if (DMA) {
#pragma unroll
        for (int i = 0; i < NC; ++i)
          ss += chunk_sumsq<T>(*reinterpret_cast<const uint4*>(
              ktile + row * RBt + ((((tid & 1) * NC + i) ^ swizzle_of_row<T, D>(row)) * 16)));
      } else {
        const uint4* p = reinterpret_cast<const uint4*>(ktile + row * TL::kStride + (tid & 1) * TL::kHalfBytes);
#pragma unroll
        for (int i = 0; i < NC; ++i) ss += chunk_sumsq<T>(p[i]);
      }
      ss += __shfl_xor(ss, 1, kWave);
      if ((tid & 1) == 0 && row < rows_valid) invn_out[j0 + row] = 1.0f / fmaxf(sqrtf(ss), 1e-30f);
    }

    for (int sb = cs; active && sb < kScoreTile / 32; sb += a.CS) {
      const int jb = j0 + sb * 32;
      if (jb >= a.T || (BLOCKS && jb > wave_last)) break;  // past the sequence, or past every row of this wave
      Frag<T, D> kf;
      uint32_t mword;
      if (DMA) {
#pragma unroll
        for (int c = 0; c < NC; ++c) kf.c[c] = *reinterpret_cast<const uint4*>(ktile + sb * 32 * RBt + coff[c]);
        mword = (uint32_t)((sb & 2 ? cur1 : cur0) >> ((sb & 1) * 32));
      } else {
        frag_load(kf, ktile + (sb * 32 + n) * TL::kStride, kg);
        mword = (uint32_t)__ballot(lmask[sb * 32 + n] != 0);
      }
      const bool tail = jb + 31 >= a.T;  // the block runs past the end of the sequence
      const bool one_modality = mword == 0u || mword == 0xffffffffu;
      const bool full_all = jb + 31 <= a.T - a.W;  // every key of the block is visible to every row of the window
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        // A fragment's 32 rows sit at the positions qlast-31 .. qlast.  With row blocks of several hundred rows
        // (BLOCKS) the 32-key block is classified per fragment: keys after qlast are invisible to all of its rows
        // (nothing to add), keys up to qlast-31 are visible to all of them (no per-element test needed).
        if (q < nvalid && (!BLOCKS || jb <= qlast[q])) {
          const bool full = BLOCKS ? (!tail && jb + 31 <= qlast[q] - 31) : full_all;
          const bool uniform = full && one_modality;
          f32x16_t acc = acc_zero();
          mma<T, D>(acc, kf, qf[q]);
          if (full) {
            // every key of the block counts: the maximum is taken on the raw products (the scale is positive, so
            // it commutes with the maximum) and the scale is folded into the exponent's multiply-add
            float bm = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
#pragma unroll
            for (int r = 3; r < 15; r += 2) bm = fmaxf(fmaxf(bm, acc[r]), acc[r + 1]);
            bm = fmaxf(bm, acc[15]);
            const float mn = fmaxf(m[q], bm * a.c);
            const float sc = fast_exp2(m[q] - mn);
            zv[q] *= sc;
            zt[q] *= sc;
            m[q] = mn;
            if (uniform) {
              float s = 0.f;
#pragma unroll
              for (int r = 0; r < 16; ++r) s += fast_exp2(fmaf(acc[r], a.c, -mn));
              if (mword)
                zv[q] += s;
              else
                zt[q] += s;
            } else {
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const float e = fast_exp2(fmaf(acc[r], a.c, -mn));
                const bool vis = (mword >> acc_row(r, kg)) & 1u;
                zv[q] += vis ? e : 0.f;
                zt[q] += vis ? 0.f : e;
              }
            }
          } else {
            float t[16];
            const int p = a.T - a.W + qrow[q];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int j = jb + acc_row(r, kg);
              t[r] = (j < a.T && j <= p) ? acc[r] * a.c : kNegBig;
            }
            float bm = t[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) bm = fmaxf(bm, t[r]);
            const float mn = fmaxf(m[q], bm);
            const float sc = fast_exp2(m[q] - mn);
            zv[q] *= sc;
            zt[q] *= sc;
            m[q] = mn;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              // the exponent in the form pass B uses (one rounding, as in the plain path above): the probability of
              // a row's largest logit is then the same number in both passes, and a nearly one-hot row keeps its
              // normaliser consistent with its probabilities
              const float e = (t[r] > 0.5f * kNegBig) ? fast_exp2(fmaf(acc[r], a.c, -mn)) : 0.f;
              const bool vis = (mword >> acc_row(r, kg)) & 1u;
              zv[q] += vis ? e : 0.f;
              zt[q] += vis ? 0.f : e;
            }
          }
        }
      }
    }
  }

  // the two lane groups hold disjoint keys of the same query row: merge them, then store the partial
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    if (q < nvalid) {
      const float mo = __shfl_xor(m[q], 32, kWave);
      const float zvo = __shfl_xor(zv[q], 32, kWave);
      const float zto = __shfl_xor(zt[q], 32, kWave);
      const float M = fmaxf(m[q], mo);
      const float f1 = fast_exp2(m[q] - M), f2 = fast_exp2(mo - M);
      if (kg == 0 && qrow[q] < a.W) {
        const size_t row_id = (size_t)(l * a.Hq + qhead[q]) * a.stats_rows + a.stats_row0 + qrow[q];
        a.stats_part[row_id * a.NPART + ch * a.CS + cs] =
            make_float4(M, zv[q] * f1 + zvo * f2, zt[q] * f1 + zto * f2, 0.f);
      }
    }
  }
}

// One thread per (layer, query head, row of the statistics arrays): merge the partials of the row.
__global__ void __launch_bounds__(256) stats_combine_kernel(ScoreArgs a) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = a.L * a.Hq * a.stats_rows;
  if (idx >= total) return;
  const int row = idx % a.stats_rows;
  const int n_part = a.NPART;
  int position;  // the row's position in the sequence
  if (a.blocks) {
    position = a.Tk - a.q_rows + row;  // one chunk of keys per row block: every partial of the row exists
  } else {
    if (row >= a.W) {  // padding rows of the window: no weight
      float* plane = reinterpret_cast<float*>(a.stats) + (size_t)(idx / a.stats_rows) * 4 * a.stats_rows + row;
      plane[0] = plane[(size_t)a.stats_rows] = plane[2 * (size_t)a.stats_rows] = plane[3 * (size_t)a.stats_rows] = 0.f;
      return;
    }
    position = a.T - a.W + row;
  }
  const float4* part = a.stats_part + (size_t)idx * a.NPART;
  float M = kNegBig;
  for (int i = 0; i < n_part; ++i) M = fmaxf(M, part[i].x);
  float zv = 0.f, zt = 0.f;
  for (int i = 0; i < n_part; ++i) {
    const float4 p = part[i];
    const float f = fast_exp2(p.x - M);
    zv = fmaf(p.y, f, zv);
    zt = fmaf(p.z, f, zt);
  }
  const int l = idx / (a.Hq * a.stats_rows);
  const bool row_is_vision = a.mask[(size_t)(l / a.Lseq) * a.Tk + position] != 0;
  const float coef_v = (!row_is_vision && zv > 0.f) ? 1.0f / zv : 0.f;  // text row: attends to vision columns
  const float coef_t = (row_is_vision && zt > 0.f) ? 1.0f / zt : 0.f;   // vision row: attends to text columns
  if (a.blocks) {
    // The statistics are stored as four planes of stats_rows values per (layer, head), so that pass B can copy the
    // values of a row block and a plane as one contiguous piece.  Row-block mode: the planes hold the form the inner
    // loop of that mode wants.  The probability of key j is
    // exp2(c * (q.k_j + bias)) with bias = -(M + log2 Z) / c, which pass B puts into the accumulators before the
    // matrix products; the cross-modal probability is that times Z / Z_cross (0 for rows of the wrong modality or
    // without cross-modal mass).
    const float z = zv + zt;
    float* plane = reinterpret_cast<float*>(a.stats) + (size_t)(idx / a.stats_rows) * 4 * a.stats_rows + row;
    plane[0] = -(M + __log2f(z)) / a.c;
    plane[(size_t)a.stats_rows] = (!row_is_vision && zv > 1e-30f) ? z / zv : 0.f;     // weight on vision columns
    plane[2 * (size_t)a.stats_rows] = (row_is_vision && zt > 1e-30f) ? z / zt : 0.f;  // weight on text columns
    plane[3 * (size_t)a.stats_rows] = 0.f;
  } else {
    // the window: row maximum, 1/Z, and the cross-modal 1/Z as the weight on vision and on text columns
    float* plane = reinterpret_cast<float*>(a.stats) + (size_t)(idx / a.stats_rows) * 4 * a.stats_rows + row;
    plane[0] = M;
    plane[(size_t)a.stats_rows] = 1.0f / (zv + zt);
    plane[2 * (size_t)a.stats_rows] = coef_v;
    plane[3 * (size_t)a.stats_rows] = coef_t;
  }
}

// ------------------------------------------------------------------------------------------ launch

template <typename T, int D, int NQ, int NW, bool BLOCKS, bool DMA>
static hipError_t launch_stats_b(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  const size_t lds = DMA ? 2 * (size_t)kScoreTile * Tile<T, D>::kRowBytes : (size_t)kScoreTile * Tile<T, D>::kStride + kScoreTile;
  auto kern = score_stats_kernel<T, D, NQ, NW, BLOCKS, DMA>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_dynamic_lds(kern, (int)lds);
    if (e != hipSuccess) return e;
  }
  dim3 grid(p.NCH, p.Hkv * p.n_blocks_a, p.L), block(NW * 64);
  hipLaunchKernelGGL(kern, grid, block, lds, s, a);
  return hipGetLastError();
}

template <typename T, int D, int NQ, int NW>
static hipError_t launch_stats_w(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  // Asynchronous copies where the pass is not already at the memory's rate: grouped heads, and every prompt row
  // scoring.  With one query head per kv head and a window of 32 rows the pass streams the keys at the rate a plain
  // read reaches, and three workgroups per CU of the small register-staged form do that best.
  constexpr bool kCanDma = Tile<T, D>::kRowBytes <= 256;
  if constexpr (kCanDma) {
    if (p.blocks) return launch_stats_b<T, D, NQ, NW, true, true>(p, a, s);
    if (p.G >= 2) return launch_stats_b<T, D, NQ, NW, false, true>(p, a, s);
  }
  return p.blocks ? launch_stats_b<T, D, NQ, NW, true, false>(p, a, s) : launch_stats_b<T, D, NQ, NW, false, false>(p, a, s);
}

template <typename T, int D, int NQ>
static hipError_t launch_stats_t(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  return p.NCG * p.CS <= 4 ? launch_stats_w<T, D, NQ, 4>(p, a, s) : launch_stats_w<T, D, NQ, 8>(p, a, s);
}

template <typename T, int D>
static hipError_t launch_stats_d(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  switch (p.NQ) {
    case 1: return launch_stats_t<T, D, 1>(p, a, s);
    case 2: return launch_stats_t<T, D, 2>(p, a, s);
    default: return launch_stats_t<T, D, 4>(p, a, s);
  }
}

hipError_t launch_score_stats(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b, true);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_stats_d<bf16_t, 128>(p, a, s) : launch_stats_d<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_stats_d<float, 128>(p, a, s) : launch_stats_d<float, 64>(p, a, s);
}

hipError_t launch_stats_combine(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b);
  const int total = p.L * p.Hq * (p.blocks ? p.R : p.Wp);
  hipLaunchKernelGGL(stats_combine_kernel, dim3((total + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace meda
