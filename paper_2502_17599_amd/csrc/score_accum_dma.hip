// Pass B of the scoring (Sections 3.2 and 3.3) for grouped query heads and observation windows of up to 96 rows: the
// arithmetic of score_accum_kernel, instruction for instruction (same products, same order of every sum, so the
// results are bit-identical), with another way of feeding it.  A workgroup walks over all query heads against one
// column tile of 128 keys; per head it needs the window's query rows and row statistics, per kv head the key tile.
// Here they come by asynchronous global-to-LDS copies (no staging registers, no LDS store instructions): the copies
// of head h+1 (and of the next kv head's key tile, when h+1 starts a new group) are issued when head h starts, so a
// head costs one wait and one barrier and no load is waited for where it is issued.
//
// One key tile buffer is enough with at least two query heads per kv head: every wave takes its key fragment out of
// the buffer in the first head of a group, and the next tile is requested in the last head of the group, at least one
// barrier later.  (With one query head per kv head score_accum_kernel stages the next tile through registers.)
//
// LDS tiles filled by the copies are unpadded and xor-swizzled (swizzle_of_row in device_utils.hpp).
// grid (NT, L) x 4 waves: wave cw owns the 32 key columns cw*32.. of the tile (a lane owns one column) and all RB
// 32-row blocks of the window.
#include "score_common.hpp"

namespace meda {

constexpr int kDmaWaves = 4;
constexpr int kDmaThreads = kDmaWaves * 64;

template <typename T, int D, int RB>
constexpr int dma_stage_bytes() {  // the window's query rows and the four planes of their statistics
  return RB * 32 * Tile<T, D>::kRowBytes + 4 * RB * 32 * (int)sizeof(float);
}

template <typename T, int D, int RB>
constexpr size_t dma_lds_bytes() {  // the key tile, two stages, the entropy reduction
  return (size_t)kScoreTile * Tile<T, D>::kRowBytes + 2 * (size_t)dma_stage_bytes<T, D, RB>() + kDmaWaves * 2 * sizeof(double);
}

template <typename T, int D, int RB>
__global__ void __launch_bounds__(kDmaThreads, 2) score_accum_dma_kernel(ScoreArgs a) {
  using TL = Tile<T, D>;
  constexpr int RBt = TL::kRowBytes;
  constexpr int CPR = TL::kChunksPerRow;
  constexpr int NC = TL::kFragChunks;
  constexpr int RPI = 64 / CPR;                          // rows one copy instruction fills
  constexpr int PFK = kScoreTile / RPI / kDmaWaves;      // key copy instructions per wave and tile
  constexpr int QI = RB * 32 / RPI;                      // copy instructions of a window of query rows
  constexpr int PFQ = (QI + kDmaWaves - 1) / kDmaWaves;  // per wave (the last ones may be beyond QI)
  constexpr int Wp = RB * 32;
  constexpr int kTileBytes = kScoreTile * RBt;
  constexpr int kQBytes = Wp * RBt;
  constexpr int kStageBytes = dma_stage_bytes<T, D, RB>();
  static_assert(64 % CPR == 0 && kScoreTile % (RPI * kDmaWaves) == 0, "the copy instructions must tile a tile evenly");
  extern __shared__ __align__(16) char smem[];  // key tile, stage 0, stage 1, reduction
  double* red = reinterpret_cast<double*>(smem + kTileBytes + 2 * kStageBytes);  // [waves][2]

  // layers are walked in the opposite order of pass A, so the keys pass A touched last (still in the
  // memory-side cache) are the first ones read here
  const int tile = blockIdx.x, l = a.L - 1 - blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int cw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j0 = tile * kScoreTile;
  const int j = j0 + cw * 32 + n;  // this lane's key column
  const bool col_ok = j < a.T;
  const bool col_is_vision = col_ok && a.mask[(size_t)(l / a.Lseq) * a.Tk + j] != 0;
  const int coef_plane = col_is_vision ? 2 : 3;
  // rows past the window (W not a multiple of 32) repeat the last query row and have zero weights; the masked path
  // also drops their exponentials, which the plain path would multiply by zero (not safe if one overflowed)
  const bool full = j0 + kScoreTile - 1 <= a.T - a.W && a.W == Wp;

  // Key copy c of this wave fills the rows (cw * PFK + c) * RPI .. + RPI-1 of the tile, query copy c the rows
  // (cw * PFQ + c) * RPI .. of the window: this lane brings one 16-byte chunk.  Key rows past the end of the sequence
  // repeat the last key (their columns are masked), query rows past the window the last row.
  unsigned koff[PFK], qoff[PFQ];
#pragma unroll
  for (int c = 0; c < PFK; ++c) {
    const int r = (cw * PFK + c) * RPI + lane / CPR;
    koff[c] = (unsigned)min(j0 + r, a.Tk - 1) * RBt + (unsigned)(((lane % CPR) ^ swizzle_of_row<T, D>(r)) * 16);
  }
#pragma unroll
  for (int c = 0; c < PFQ; ++c) {
    const int r = (cw * PFQ + c) * RPI + lane / CPR;
    qoff[c] = (unsigned)(a.q_row0 + min(r, a.W - 1)) * RBt + (unsigned)(((lane % CPR) ^ swizzle_of_row<T, D>(r)) * 16);
  }
  const unsigned lds0 = (unsigned)(size_t)smem;
  const float* stats_f = reinterpret_cast<const float*>(a.stats);
  auto issue = [&](int h) {
    const int g = h / a.G;
    const unsigned stage = lds0 + (unsigned)(kTileBytes + (h & 1) * kStageBytes);
    if (h - g * a.G == 0) {
      const char* ksrc = uniform_ptr(a.k + (size_t)(l * a.Hkv + g) * a.Tk * RBt);
#pragma unroll
      for (int c = 0; c < PFK; ++c) async_copy16_to_lds_stream(ksrc, koff[c], lds0 + (unsigned)((cw * PFK + c) * 1024));
    }
    const char* qsrc = uniform_ptr(a.q + (size_t)(l * a.Hq + h) * a.q_rows * RBt);
#pragma unroll
    for (int c = 0; c < PFQ; ++c)
      if (cw * PFQ + c < QI) async_copy16_to_lds(qsrc, qoff[c], stage + (unsigned)((cw * PFQ + c) * 1024));
    // the 4 * Wp statistics of the head are contiguous: wave w brings the values w*64 .. w*64+63 of them
    const float* ssrc = uniform_ptr(stats_f + (size_t)(l * a.Hq + h) * 4 * Wp);
#pragma unroll
    for (int w0 = 0; w0 < 4 * Wp; w0 += kDmaThreads)
      if (w0 + cw * 64 < 4 * Wp)
        async_copy4_to_lds(ssrc, (unsigned)(w0 + cw * 64 + lane) * 4u,
                           stage + (unsigned)(kQBytes + (w0 + cw * 64) * 4));
  };

  // chunk c of this lane's fragment (chunk kg * NC + c of row n of a 32-row block) sits at (n * row bytes) +
  // 16 * ((kg * NC + c) ^ swz(n)) inside the block; the swizzle of a row does not depend on its block
  unsigned coff[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) coff[c] = (unsigned)(n * RBt + (((kg * NC + c) ^ swizzle_of_row<T, D>(n)) * 16));
  auto frag_from = [&](Frag<T, D>& f, const char* block) {
#pragma unroll
    for (int c = 0; c < NC; ++c) f.c[c] = *reinterpret_cast<const uint4*>(block + coff[c]);
  };

  float pbar[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) pbar[rb][r] = 0.f;
  Frag<T, D> kf;
  float colsum = 0.f;

  issue(0);
  for (int h = 0; h < a.Hq; ++h) {
    async_copy_wait<0>();  // this wave's pieces of the head have landed
    __syncthreads();       // every wave's have; and nobody reads the other stage (the previous head) any more
    if (h + 1 < a.Hq) issue(h + 1);
    const int g = h / a.G, hg = h - g * a.G;
    const char* stage = smem + kTileBytes + (h & 1) * kStageBytes;
    const float* st = reinterpret_cast<const float*>(stage + kQBytes);  // planes: maximum, 1/Z, the two cross-modal 1/Z
    if (hg == 0) {
      frag_from(kf, smem + cw * 32 * RBt);  // the key tile of this kv head
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
      for (int rb = 0; rb < RB; ++rb) {
        Frag<T, D> qf;
        frag_from(qf, stage + rb * 32 * RBt);
        f32x16_t acc = acc_zero();
        mma<T, D>(acc, qf, kf);
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int row0 = rb * 32 + r4 * 8 + kg * 4;  // rows of acc[r4*4 .. r4*4+3]
          const float4 m4 = *reinterpret_cast<const float4*>(st + row0);
          const float4 z4 = *reinterpret_cast<const float4*>(st + Wp + row0);
          const float4 c4 = *reinterpret_cast<const float4*>(st + coef_plane * Wp + row0);
          const float mm[4] = {m4.x, m4.y, m4.z, m4.w};
          const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
          const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float e = fast_exp2(fmaf(acc[r4 * 4 + i], a.c, -mm[i]));
            if (MASKED) e = (rb * 32 + r4 * 8 + i >= row_min && rb * 32 + r4 * 8 + i < row_end) ? e : 0.f;
            colsum = fmaf(e, zz[i], colsum);
            pbar[rb][r4 * 4 + i] = fmaf(e, cc[i], pbar[rb][r4 * 4 + i]);
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
      if (kg == 0 && col_ok) a.col_scores[(size_t)(l * a.Hkv + g) * a.Tk + j] = tot;  // one writer per column
    }
  }

  // entropy terms of the head-averaged cross-modal probabilities.  A vision column only receives
  // probability from text rows (text -> vision direction) and a text column only from vision rows.
  const float inv_heads = 1.0f / (float)a.Hq;
  float s = 0.f;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = pbar[rb][r] * inv_heads;
      s += (p > 0.f) ? p * __logf(p) : 0.f;
    }
  const double tv = wave_sum(col_is_vision ? (double)s : 0.0);
  const double vt = wave_sum((col_ok && !col_is_vision) ? (double)s : 0.0);
  if (lane == 0) {
    red[cw * 2 + 0] = tv;
    red[cw * 2 + 1] = vt;
  }
  __syncthreads();
  if (tid < 2) {
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < kDmaWaves; ++w) sum += red[w * 2 + tid];
    a.ent_part[((size_t)l * a.NTk + tile) * 2 + tid] = -sum;
  }
}

// ------------------------------------------------------------------------------------------ launch

template <typename T, int D, int RB>
static hipError_t launch_dma_k(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  constexpr size_t lds = dma_lds_bytes<T, D, RB>();
  auto kern = score_accum_dma_kernel<T, D, RB>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_dynamic_lds(kern, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(p.NT, p.L), dim3(kDmaThreads), lds, s, a);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_dma_t(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  switch (p.RB) {
    case 1: return launch_dma_k<T, D, 1>(p, a, s);
    case 2: return launch_dma_k<T, D, 2>(p, a, s);
    default: return launch_dma_k<T, D, 3>(p, a, s);
  }
}

// Grouped heads (one key tile buffer), windows of at most three 32-row blocks (four waves), rows of at most 256
// bytes (two stages fit twice per CU).
bool score_accum_dma_supported(const Plan& p) {
  return !p.blocks && p.accumulate == 0 && p.G >= 2 && p.RB <= 3 && p.d * p.elt <= 256;
}

hipError_t launch_score_accum_dma(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_dma_t<bf16_t, 128>(p, a, s) : launch_dma_t<bf16_t, 64>(p, a, s);
  return launch_dma_t<float, 64>(p, a, s);
}

}  // namespace meda
