// Pass B of the scoring (Sections 3.2 and 3.3): with the row statistics of pass A, the probabilities are formed
// again and added into the column scores A_s and into the head-averaged cross-modal matrix, whose entropy terms are
// reduced per column tile.  The layout of the pass is described in score_common.hpp.
#include "score_common.hpp"

namespace meda {

// ------------------------------------------------------------------------------------------ pass B
// grid (NT, L); NW = 4 or 8 waves.  Wave (cw, rh) = (wave & 3, wave >> 2) owns the 32 key columns cw*32.. of
// the tile (a lane owns one column) and the row blocks rh*RBW .. rh*RBW + RBW-1 of the window, RBW = RB / (NW/4).
// The workgroup walks over all kv heads and, inside, the query heads of the group, so the
// head-averaged cross-modal probabilities of its W x 128 patch accumulate in registers (same
// accumulator layout for every head) and the entropy terms p log p can be taken once at the end.
// Eight waves (two per SIMD, each with half of the rows) let one wave's exponentials run beside the
// other's matrix products; they are used when a wave would otherwise hold several row blocks.
template <typename T, int D, int RB, bool KSTAGE, int NW, bool BLOCKS>
__global__ void __launch_bounds__(NW * 64, (NW == 8) ? 2 : ((RB == 1 && sizeof(T) == 2 && !KSTAGE) ? 3 : 1))
    score_accum_kernel(ScoreArgs a0) {
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
  int tile = blockIdx.x, l = a0.L - 1 - blockIdx.y;
  if (BLOCKS) {
    // Row-block mode (more than 128 scoring rows): the workgroup takes its column tile through ALL row blocks that see it (block bi
    // sees the tile iff j0 < Tk - bi * row_block), one after the other: one writer per column and entropy partial,
    // in a fixed order, so the sums do not depend on the launch.  Tile t is seen by NT - t row blocks: the longest
    // workgroups go first (tile 0 of all layers, then tile 1, ...).  (Giving a workgroup the tiles t and NT-1-t, and
    // each XCD whole layers so that its workgroups share query blocks in L2, was measured: more L2 hits, but slower.)
    const int id = blockIdx.y * gridDim.x + blockIdx.x;
    tile = id / a0.L;
    l = a0.L - 1 - (id - tile * a0.L);
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int cw = wave & 3, rh = wave >> 2;
  const int j0 = tile * kScoreTile;
  const int j = j0 + cw * 32 + n;  // this lane's key column
  // statistics of row `row` of the launch's (or the block's) rows, head index lh = l * Hq + h
  auto load_row_stats = [&](const ScoreArgs& a, int lh, int row) {
    // four planes of stats_rows values per (layer, head), written by stats_combine_kernel
    const float* plane = reinterpret_cast<const float*>(a.stats) + (size_t)lh * 4 * a.stats_rows + a.stats_row0 + row;
    const size_t ps = (size_t)a.stats_rows;
    // every prompt row scores: the bias of the logits and the weights of the cross-modal probabilities on vision
    // and on text columns; the probability itself has weight 1
    if (BLOCKS) return make_float4(plane[0], 1.0f, plane[ps], plane[2 * ps]);
    return make_float4(plane[0], plane[ps], plane[2 * ps], plane[3 * ps]);  // maximum, 1/Z, the two cross-modal 1/Z
  };
  auto one_block = [&](const ScoreArgs& a) {
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
  const float4 no_stats = make_float4(0.f, 0.f, 0.f, 0.f);  // rows past the block: zero queries, zero weights
  sreg = no_stats;
  if (tid < a.W) sreg = load_row_stats(a, l * a.Hq, tid);

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
      sreg = no_stats;
      if (tid < a.W) sreg = load_row_stats(a, l * a.Hq + hn, tid);
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
#pragma unroll(BLOCKS ? 1 : RBW)
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
            float e = BLOCKS ? fast_exp2((acc[r4 * 4 + i] + mm[i]) * a.c) : fast_exp2(fmaf(acc[r4 * 4 + i], a.c, -mm[i]));
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
  };
  if (!BLOCKS) {
    one_block(a0);
  } else {
    // row blocks that exist and see this tile
    const int n_bi = min((a0.Tk - j0 + a0.row_block - 1) / a0.row_block, (a0.q_rows + a0.row_block - 1) / a0.row_block);
    for (int bi = 0; bi < n_bi; ++bi) {
      ScoreArgs a = a0;
      select_row_block(a, bi);
      __syncthreads();  // the previous row block's tiles and sums are no longer read
      one_block(a);
    }
  }
}

// ------------------------------------------------------------------------------------------ launch

template <typename T, int D, int RB, bool KSTAGE, int NW, bool BLOCKS = false>
static hipError_t launch_accum_k(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  const size_t lds = (size_t)(kScoreTile + RB * 32) * Tile<T, D>::kStride + (4 * RB * 32 + kScoreTile) * sizeof(float) +
                     NW * 2 * sizeof(double);
  auto kern = score_accum_kernel<T, D, RB, KSTAGE, NW, BLOCKS>;
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
  if constexpr (RB == kScoreRowBlock / 32) {
    if (p.blocks) {  // row-block mode: row blocks walked inside the kernel
      if (p.G == 1) return launch_accum_k<T, D, RB, true, NW, true>(p, a, s);
      return launch_accum_k<T, D, RB, false, NW, true>(p, a, s);
    }
  }
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
  if (score_accum_blocks_supported(p)) return launch_score_accum_blocks(p, b, s);
  if (score_accum_dma_supported(p)) return launch_score_accum_dma(p, b, s);
  const ScoreArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_accum_d<bf16_t, 128>(p, a, s) : launch_accum_d<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_accum_d<float, 128>(p, a, s) : launch_accum_d<float, 64>(p, a, s);
}

}  // namespace meda
