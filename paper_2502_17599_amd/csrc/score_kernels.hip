// Scoring phases of the compression pass (Section 3.2: cross-modal attention entropy; Section 3.3:
// cumulative attention score).  The softmax normalisers of a window row are needed before any of its
// probabilities can be added to a column sum or to the head-averaged cross-modal matrix, so the keys
// are visited twice:
//   pass A  score_stats_kernel   row maxima and normalisers (all keys / vision keys / text keys),
//                                split over column chunks; also 1/|k| of every key (used by the merge)
//           stats_combine_kernel merges the chunk partials of every row
//   pass B  score_accum_kernel   recomputes the logits, adds normalised probabilities into the column
//                                scores A_s and into the head-averaged cross-modal matrix, whose row
//                                entropies are reduced per tile
// Logits are kept in the base-2 domain: t = (q.k) * scale * log2(e), probabilities are exp2(t - max).
#include <type_traits>

#include "device_utils.hpp"
#include "plan.hpp"

namespace meda {

struct ScoreArgs {
  const char* q;
  const char* k;
  const uint8_t* mask;  // [N][Tk]: layer l belongs to sequence l / Lseq
  float4* stats_part;  // [L][Hq][Wp][NPART] (max, Z_vision, Z_text, -)
  float4* stats;       // [L][Hq][Wp]        (max, 1/Z_all, coef for vision columns, coef for text columns)
  float* inv_norm;     // [L][Hkv][T]
  float* col_scores;   // [L][Hkv][T]
  double* ent_part;    // [L][NT][2]
  int L, Hq, Hkv, G, T, W, RB, Wp;   // T keys and W query rows of this launch (the last W positions below T)
  int Lseq;        // layers per sequence
  int NCG, CS, CH, NPART, NT;
  int Tk;          // key rows per (layer, kv head) in memory (>= T)
  int q_rows;      // rows per (layer, head) in the query buffer
  int q_row0;      // first query row of this launch in the buffer
  int NTk;         // tiles per layer in ent_part
  int accumulate;  // add to col_scores / ent_part instead of storing
  float c;             // scale * log2(e)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------------------------------ pass A
// grid (NCH, Hkv, L); NCG*CS waves.  Wave (cg, cs) keeps NQ query fragments ((head of the group, row
// block) pairs cg*NQ .. cg*NQ+NQ-1) in registers and visits the 32-key blocks sb = cs, cs+CS, ... of
// every tile of its chunk.  The product is taken with the keys as operand A and the queries as
// operand B, so a lane owns one query row and 16 keys per block: the running (max, Z_vision, Z_text)
// of the row live in three registers per fragment and need no cross-lane traffic until the end.
template <typename T, int D, int NQ, int NW>
__global__ void __launch_bounds__(NW * 64, (NQ == 1 && NW == 4 && sizeof(T) == 2) ? 3 : 2) score_stats_kernel(ScoreArgs a) {
  using TL = Tile<T, D>;
  extern __shared__ __align__(16) char smem[];
  char* ktile = smem;
  uint8_t* lmask = reinterpret_cast<uint8_t*>(smem + kScoreTile * TL::kStride);

  const int ch = blockIdx.x, g = blockIdx.y, l = blockIdx.z;
  constexpr int nthr = NW * 64;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int cgi = wave % a.NCG, cs = wave / a.NCG;
  const bool active = cs < a.CS;  // the workgroup is padded to 4 or 8 waves; spare waves only move data
  const int n_combos = a.G * a.RB;

  Frag<T, D> qf[NQ];
  float m[NQ], zv[NQ], zt[NQ];
  int qrow[NQ], qhead[NQ];
  int nvalid = 0;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int cidx = cgi * NQ + q;
    m[q] = kNegBig;
    zv[q] = 0.f;
    zt[q] = 0.f;
    qrow[q] = 0;
    qhead[q] = 0;
    frag_zero(qf[q]);
    if (active && cidx < n_combos) {
      nvalid = q + 1;
      const int hg = cidx / a.RB, rb = cidx - hg * a.RB;
      qhead[q] = g * a.G + hg;
      qrow[q] = rb * 32 + n;
      if (qrow[q] < a.W)
        frag_load(qf[q], a.q + ((size_t)(l * a.Hq + qhead[q]) * a.q_rows + a.q_row0 + qrow[q]) * TL::kRowBytes, kg);
    }
  }

  const uint8_t* mask = a.mask + (size_t)(l / a.Lseq) * a.Tk;  // this layer's sequence
  const int jbeg = ch * a.CH;
  const int jend = min(a.T, jbeg + a.CH);
  const char* kbase = a.k + (size_t)(l * a.Hkv + g) * a.Tk * TL::kRowBytes;
  float* invn_out = a.inv_norm + (size_t)(l * a.Hkv + g) * a.Tk;

  TileStage<T, D, kScoreTile, nthr> stage;
  uint8_t mreg = 0;
  if (jbeg < jend) {
    stage.template fetch<true>(kbase + (size_t)jbeg * TL::kRowBytes, min(kScoreTile, a.T - jbeg), tid, nthr);
    if (tid < kScoreTile) mreg = (jbeg + tid < a.T) ? mask[jbeg + tid] : 0;
  }
  for (int j0 = jbeg; j0 < jend; j0 += kScoreTile) {
    __syncthreads();  // the previous tile is no longer read
    const int rows_valid = min(kScoreTile, a.T - j0);
    stage.commit(ktile, tid, nthr);
    if (tid < kScoreTile) lmask[tid] = mreg;
    __syncthreads();
    if (j0 + kScoreTile < jend) {  // next tile's loads are in flight while this one is processed
      const int jn = j0 + kScoreTile;
      stage.template fetch<true>(kbase + (size_t)jn * TL::kRowBytes, min(kScoreTile, a.T - jn), tid, nthr);
      if (tid < kScoreTile) mreg = (jn + tid < a.T) ? mask[jn + tid] : 0;
    }

    // 1/|k| of the tile's keys: two threads per row
    for (int row = tid >> 1; row < kScoreTile; row += nthr >> 1) {
      const uint4* p = reinterpret_cast<const uint4*>(ktile + row * TL::kStride + (tid & 1) * TL::kHalfBytes);
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < TL::kFragChunks; ++i) ss += chunk_sumsq<T>(p[i]);
      ss += __shfl_xor(ss, 1, kWave);
      if ((tid & 1) == 0 && row < rows_valid) invn_out[j0 + row] = 1.0f / fmaxf(sqrtf(ss), 1e-30f);
    }

    for (int sb = cs; active && sb < kScoreTile / 32; sb += a.CS) {
      const int jb = j0 + sb * 32;
      if (jb >= a.T) break;
      Frag<T, D> kf;
      frag_load(kf, ktile + (sb * 32 + n) * TL::kStride, kg);
      const uint32_t mword = (uint32_t)__ballot(lmask[sb * 32 + n] != 0);
      const bool full = jb + 31 <= a.T - a.W;  // every key of the block is visible to every window row
      const bool uniform = full && (mword == 0u || mword == 0xffffffffu);
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        if (q < nvalid) {
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
              const float e = (t[r] > 0.5f * kNegBig) ? fast_exp2(t[r] - mn) : 0.f;
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
        const size_t row_id = (size_t)(l * a.Hq + qhead[q]) * a.Wp + qrow[q];
        a.stats_part[row_id * a.NPART + ch * a.CS + cs] =
            make_float4(M, zv[q] * f1 + zvo * f2, zt[q] * f1 + zto * f2, 0.f);
      }
    }
  }
}

// One thread per (layer, query head, padded window row): merge the NPART partials.
__global__ void __launch_bounds__(256) stats_combine_kernel(ScoreArgs a) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = a.L * a.Hq * a.Wp;
  if (idx >= total) return;
  const int row = idx % a.Wp;
  if (row >= a.W) {
    a.stats[idx] = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const float4* part = a.stats_part + (size_t)idx * a.NPART;
  float M = kNegBig;
  for (int i = 0; i < a.NPART; ++i) M = fmaxf(M, part[i].x);
  float zv = 0.f, zt = 0.f;
  for (int i = 0; i < a.NPART; ++i) {
    const float4 p = part[i];
    const float f = fast_exp2(p.x - M);
    zv = fmaf(p.y, f, zv);
    zt = fmaf(p.z, f, zt);
  }
  const int l = idx / (a.Hq * a.Wp);
  const bool row_is_vision = a.mask[(size_t)(l / a.Lseq) * a.Tk + a.T - a.W + row] != 0;
  const float coef_v = (!row_is_vision && zv > 0.f) ? 1.0f / zv : 0.f;  // text row: attends to vision columns
  const float coef_t = (row_is_vision && zt > 0.f) ? 1.0f / zt : 0.f;   // vision row: attends to text columns
  a.stats[idx] = make_float4(M, 1.0f / (zv + zt), coef_v, coef_t);
}

// ------------------------------------------------------------------------------------------ pass B
// grid (NT, L); NW = 4 or 8 waves.  Wave (cw, rh) = (wave & 3, wave >> 2) owns the 32 key columns cw*32.. of
// the tile (a lane owns one column) and the row blocks rh*RBW .. rh*RBW + RBW-1 of the window, RBW = RB / (NW/4).
// The workgroup walks over all kv heads and, inside, the query heads of the group, so the
// head-averaged cross-modal probabilities of its W x 128 patch accumulate in registers (same
// accumulator layout for every head) and the entropy terms p log p can be taken once at the end.
// Eight waves (two per SIMD, each with half of the rows) let one wave's exponentials run beside the
// other's matrix products; they are used when a wave would otherwise hold several row blocks.
template <typename T, int D, int RB, bool KSTAGE, int NW>
__global__ void __launch_bounds__(NW * 64, (NW == 8) ? 2 : ((RB == 1 && sizeof(T) == 2 && !KSTAGE) ? 3 : 1))
    score_accum_kernel(ScoreArgs a) {
  using TL = Tile<T, D>;
  constexpr int NTHR = NW * 64;
  constexpr int NRH = NW / 4;     // row groups of the workgroup
  constexpr int RBW = RB / NRH;   // row blocks per wave
  static_assert(RB % NRH == 0, "row blocks must split evenly over the row groups");
  extern __shared__ __align__(16) char smem[];
  char* ktile = smem;
  char* qtile = ktile + kScoreTile * TL::kStride;
  float* st_m = reinterpret_cast<float*>(qtile + RB * 32 * TL::kStride);
  float* st_rz = st_m + RB * 32;
  float* st_cv = st_rz + RB * 32;
  float* st_ct = st_cv + RB * 32;
  float* colred = st_ct + RB * 32;                                  // [kScoreTile] column sums of the second row group
  double* red = reinterpret_cast<double*>(colred + kScoreTile);     // [NW][2]

  // layers are walked in the opposite order of pass A, so the keys pass A touched last (still in the
  // memory-side cache) are the first ones read here
  const int tile = blockIdx.x, l = a.L - 1 - blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int cw = wave & 3, rh = wave >> 2;
  const int j0 = tile * kScoreTile;
  const int j = j0 + cw * 32 + n;  // this lane's key column
  const bool col_ok = j < a.T;
  const bool col_is_vision = col_ok && a.mask[(size_t)(l / a.Lseq) * a.Tk + j] != 0;
  const float* st_coef = col_is_vision ? st_cv : st_ct;
  const bool full = j0 + kScoreTile - 1 <= a.T - a.W;
  const int rows_valid = min(kScoreTile, a.T - j0);
  const int Wp = RB * 32;

  float pbar[RBW][16];
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) pbar[rb][r] = 0.f;

  // Heads are visited in order h = 0 .. Hq-1 (kv head g = h / G).  The tiles of head h+1 are fetched
  // into registers while head h is processed out of LDS.  With grouped heads (KSTAGE false) the key
  // tile changes only every G heads: it is then loaded on the spot, which keeps 32 registers free
  // (two waves per SIMD instead of one) at the price of one exposed load per group.
  TileStage<T, D, KSTAGE ? kScoreTile : 1, NTHR> kstage;
  TileStage<T, D, RB * 32, NTHR> qstage;
  float4 sreg = make_float4(0.f, 0.f, 0.f, 0.f);
  const char* ktile_src = a.k + ((size_t)l * a.Hkv * a.Tk + j0) * TL::kRowBytes;
  const size_t khead_stride = (size_t)a.Tk * TL::kRowBytes;
  if (KSTAGE) kstage.template fetch<true>(ktile_src, rows_valid, tid, NTHR);
  qstage.fetch(a.q + ((size_t)(l * a.Hq) * a.q_rows + a.q_row0) * TL::kRowBytes, a.W, tid, NTHR);
  if (tid < Wp) sreg = a.stats[(size_t)(l * a.Hq) * a.Wp + tid];

  Frag<T, D> kf;
  float colsum = 0.f;
  float pending = 0.f;   // column sum of a finished kv head, waiting for the other row group's share
  int pending_g = -1;
  // Adds the second row group's share (left in colred before the last barrier) and writes the column score.
  auto flush_pending = [&]() {
    if (NRH > 1 && pending_g >= 0 && rh == 0 && kg == 0 && col_ok) {
      const float tot = pending + colred[cw * 32 + n];
      float* dst = a.col_scores + (size_t)(l * a.Hkv + pending_g) * a.Tk + j;
      *dst = a.accumulate ? *dst + tot : tot;  // one writer per column and launch
    }
    pending_g = -1;
  };
  for (int h = 0; h < a.Hq; ++h) {
    const int g = h / a.G, hg = h - g * a.G;
    __syncthreads();  // the previous head's tiles are no longer read
    if (NRH > 1) flush_pending();
    if (hg == 0) {
      if (KSTAGE) {
        kstage.commit(ktile, tid, NTHR);
      } else {
        TileStage<T, D, kScoreTile, NTHR> now;
        now.template fetch<true>(ktile_src + (size_t)g * khead_stride, rows_valid, tid, NTHR);
        now.commit(ktile, tid, NTHR);
      }
    }
    qstage.commit(qtile, tid, NTHR);
    if (tid < Wp) {
      st_m[tid] = sreg.x;
      st_rz[tid] = sreg.y;
      st_cv[tid] = sreg.z;
      st_ct[tid] = sreg.w;
    }
    __syncthreads();
    if (h + 1 < a.Hq) {
      const int hn = h + 1;
      if (KSTAGE && hn % a.G == 0) kstage.template fetch<true>(ktile_src + (size_t)(hn / a.G) * khead_stride, rows_valid, tid, NTHR);
      qstage.fetch(a.q + ((size_t)(l * a.Hq + hn) * a.q_rows + a.q_row0) * TL::kRowBytes, a.W, tid, NTHR);
      if (tid < Wp) sreg = a.stats[(size_t)(l * a.Hq + hn) * a.Wp + tid];
    }
    if (hg == 0) {
      frag_load(kf, ktile + (cw * 32 + n) * TL::kStride, kg);
      colsum = 0.f;
    }
    // One query head against the wave's key columns.  MASKED: the tile touches the causal diagonal or the end
    // of the sequence, so every probability is checked against its row; all other tiles take the plain path.
    auto head_block = [&](auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      // Row r (without the lane group's offset kg*4) counts for this lane's column iff row_min <= r < row_end:
      // the row exists (r + kg*4 < W) and sees the column (j <= T - W + r + kg*4).  The bounds are made opaque
      // here so that the 16 comparisons per row block are redone per head instead of being kept in registers.
      int row_min = col_ok ? j - (a.T - a.W) - kg * 4 : (1 << 30);
      int row_end = a.W - kg * 4;
      if (MASKED) asm volatile("" : "+v"(row_min), "+v"(row_end));
#pragma unroll
      for (int rbl = 0; rbl < RBW; ++rbl) {
        const int rb = rh * RBW + rbl;
        Frag<T, D> qf;
        frag_load(qf, qtile + (rb * 32 + n) * TL::kStride, kg);
        f32x16_t acc = acc_zero();
        mma<T, D>(acc, qf, kf);
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int row0 = rb * 32 + r4 * 8 + kg * 4;  // rows of acc[r4*4 .. r4*4+3]
          const float4 m4 = *reinterpret_cast<const float4*>(st_m + row0);
          const float4 z4 = *reinterpret_cast<const float4*>(st_rz + row0);
          const float4 c4 = *reinterpret_cast<const float4*>(st_coef + row0);
          const float mm[4] = {m4.x, m4.y, m4.z, m4.w};
          const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
          const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float e = fast_exp2(fmaf(acc[r4 * 4 + i], a.c, -mm[i]));
            if (MASKED) e = (rb * 32 + r4 * 8 + i >= row_min && rb * 32 + r4 * 8 + i < row_end) ? e : 0.f;
            colsum = fmaf(e, zz[i], colsum);
            pbar[rbl][r4 * 4 + i] = fmaf(e, cc[i], pbar[rbl][r4 * 4 + i]);
          }
        }
      }
    };
    if (full)
      head_block(std::false_type{});
    else
      head_block(std::true_type{});
    if (hg == a.G - 1) {
      const float tot = colsum + __shfl_xor(colsum, 32, kWave);
      if (NRH == 1) {
        if (kg == 0 && col_ok) {
          float* dst = a.col_scores + (size_t)(l * a.Hkv + g) * a.Tk + j;
          *dst = a.accumulate ? *dst + tot : tot;  // one writer per column and launch
        }
      } else {
        if (rh == 1 && kg == 0) colred[cw * 32 + n] = tot;  // read after the next barrier
        pending = tot;
        pending_g = g;
      }
    }
  }
  if (NRH > 1) {
    __syncthreads();
    flush_pending();
  }

  // entropy terms of the head-averaged cross-modal probabilities.  A vision column only receives
  // probability from text rows (text -> vision direction) and a text column only from vision rows.
  const float inv_heads = 1.0f / (float)a.Hq;
  float s = 0.f;
#pragma unroll
  for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = pbar[rb][r] * inv_heads;
      s += (p > 0.f) ? p * __logf(p) : 0.f;
    }
  const double tv = wave_sum(col_is_vision ? (double)s : 0.0);
  const double vt = wave_sum((col_ok && !col_is_vision) ? (double)s : 0.0);
  if (lane == 0) {
    red[wave * 2 + 0] = tv;
    red[wave * 2 + 1] = vt;
  }
  __syncthreads();
  if (tid < 2) {
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red[w * 2 + tid];
    double* dst = a.ent_part + ((size_t)l * a.NTk + tile) * 2 + tid;
    *dst = a.accumulate ? *dst - sum : -sum;
  }
}

// ------------------------------------------------------------------------------------------ launch

static ScoreArgs make_args(const Plan& p, const Buffers& b) {
  ScoreArgs a;
  a.q = static_cast<const char*>(b.q);
  a.k = static_cast<const char*>(b.k);
  a.mask = b.mask;
  a.stats_part = reinterpret_cast<float4*>(b.ws + p.off_stats_part);
  a.stats = reinterpret_cast<float4*>(b.ws + p.off_stats);
  a.inv_norm = reinterpret_cast<float*>(b.ws + p.off_inv_norm);
  a.col_scores = reinterpret_cast<float*>(b.ws + p.off_col_scores);
  a.ent_part = reinterpret_cast<double*>(b.ws + p.off_ent_part);
  a.L = p.L; a.Hq = p.Hq; a.Hkv = p.Hkv; a.G = p.G; a.T = p.Tb; a.W = p.Wb; a.RB = p.RB; a.Wp = p.Wp;
  a.Lseq = p.Lseq; a.Tk = p.Tk; a.q_rows = p.R; a.q_row0 = p.q_row0; a.NTk = p.NTk; a.accumulate = p.accumulate;
  a.NCG = p.NCG; a.CS = p.CS; a.CH = p.CH; a.NPART = p.NPART; a.NT = p.NT;
  a.c = p.scale_log2;
  return a;
}

template <typename T, int D, int NQ, int NW>
static hipError_t launch_stats_w(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  const size_t lds = (size_t)kScoreTile * Tile<T, D>::kStride + kScoreTile;
  auto kern = score_stats_kernel<T, D, NQ, NW>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_dynamic_lds(kern, (int)lds);
    if (e != hipSuccess) return e;
  }
  dim3 grid(p.NCH, p.Hkv, p.L), block(NW * 64);
  hipLaunchKernelGGL(kern, grid, block, lds, s, a);
  return hipGetLastError();
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
  const ScoreArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_stats_d<bf16_t, 128>(p, a, s) : launch_stats_d<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_stats_d<float, 128>(p, a, s) : launch_stats_d<float, 64>(p, a, s);
}

hipError_t launch_stats_combine(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b);
  const int total = p.L * p.Hq * p.Wp;
  hipLaunchKernelGGL(stats_combine_kernel, dim3((total + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

template <typename T, int D, int RB, bool KSTAGE, int NW>
static hipError_t launch_accum_k(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  const size_t lds = (size_t)(kScoreTile + RB * 32) * Tile<T, D>::kStride + (4 * RB * 32 + kScoreTile) * sizeof(float) +
                     NW * 2 * sizeof(double);
  auto kern = score_accum_kernel<T, D, RB, KSTAGE, NW>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_dynamic_lds(kern, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(p.NT, p.L), dim3(NW * 64), lds, s, a);
  return hipGetLastError();
}

template <typename T, int D, int RB>
static hipError_t launch_accum_t(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  // Staging the next head's key tile through registers pays when every head brings a new key tile
  // (G == 1), except for the smallest shape, where the registers buy a third workgroup per CU instead.
  constexpr bool kThreeGroups = RB == 1 && sizeof(T) == 2;
  constexpr int NW = RB == 4 ? 8 : 4;  // four row blocks: two row groups of two (measured: no gain for two row blocks)
  if (p.G == 1 && !kThreeGroups) return launch_accum_k<T, D, RB, true, NW>(p, a, s);
  return launch_accum_k<T, D, RB, false, NW>(p, a, s);
}

template <typename T, int D>
static hipError_t launch_accum_d(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  switch (p.RB) {
    case 1: return launch_accum_t<T, D, 1>(p, a, s);
    case 2: return launch_accum_t<T, D, 2>(p, a, s);
    case 3: return launch_accum_t<T, D, 3>(p, a, s);
    default: return launch_accum_t<T, D, 4>(p, a, s);
  }
}

hipError_t launch_score_accum(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_accum_d<bf16_t, 128>(p, a, s) : launch_accum_d<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_accum_d<float, 128>(p, a, s) : launch_accum_d<float, 64>(p, a, s);
}

}  // namespace meda
