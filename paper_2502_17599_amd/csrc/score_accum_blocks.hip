// Pass B of the scoring in the row-block mode: more than 128 scoring rows, that is a long observation window or every
// prompt row (Sections 3.2 and 3.3 as the paper writes them: the column scores sum A_p over all prompt rows, the
// cross-modal matrices take all text / vision queries).  Same arithmetic as
// score_accum_kernel in its row-block mode, other data movement: the work of a workgroup is a long sequence of
// (row block, query head) items against one column tile of 128 keys, and what limits it is how the key tile, the
// query rows and the row statistics of an item get into LDS.  Here they come by asynchronous global-to-LDS copies:
// a row block has 256 rows and is taken in two halves of 128; the copies of the next half (32 KB of queries, 2 KB of
// statistics, and the next key tile when the kv head changes) are issued when a half starts, so a half costs one
// wait and one barrier, no staging registers and no LDS store instructions, and a key tile is fetched once per 256
// rows.
//
// Workgroup: 8 waves.  Wave (cw, rh) = (wave & 3, wave >> 2) owns the 32 key columns cw*32.. of the tile (a lane
// owns one column) and the rows rh*64 .. rh*64+63 of each half (two fragments of 32 rows).  The head-averaged
// cross-modal probabilities of the 256 x 128 patch stay in accumulator registers over the heads of a row block (which
// is why the row block is the outer loop and the head the inner one); their entropy terms are taken when the block
// ends.  The column sums of a kv head go to an LDS array [Hkv][128] that the workgroup alone adds to, in a fixed
// order, and that is written out once at the end: no read-modify-write of global memory, deterministic sums.
//
// LDS tiles filled by the copies are unpadded and xor-swizzled (swizzle_of_row in device_utils.hpp).
#include "score_common.hpp"

namespace meda {

constexpr int kBlkWaves = 8;
constexpr int kBlkThreads = kBlkWaves * 64;

constexpr int kBlkHalf = 128;            // rows of a half: what the waves of a workgroup cover at once
constexpr int kBlkRows = 2 * kBlkHalf;   // rows of a row block of this kernel (counted from the end of the prompt)

template <typename T, int D>
constexpr int blocks_stage_bytes() {  // one half: its query rows and four planes of row statistics (three in use)
  return kBlkHalf * Tile<T, D>::kRowBytes + 4 * kBlkHalf * (int)sizeof(float);
}

// one key tile, two stages, the column sums, the second row group's share (two buffers), the entropy reduction
template <typename T, int D>
static size_t blocks_lds_bytes(int Hkv) {
  return (size_t)kScoreTile * Tile<T, D>::kRowBytes + 2 * (size_t)blocks_stage_bytes<T, D>() +
         (size_t)Hkv * kScoreTile * sizeof(float) + 2 * kScoreTile * sizeof(float) + kBlkWaves * 2 * sizeof(double);
}

template <typename T, int D>
__global__ void __launch_bounds__(kBlkThreads, 2) score_accum_blocks_kernel(ScoreArgs a) {
  using TL = Tile<T, D>;
  static_assert(kScoreTile == 128 && kBlkHalf == 128, "the wave layout assumes 128 x 128 patches");
  constexpr int RBt = TL::kRowBytes;
  constexpr int CPR = TL::kChunksPerRow;
  constexpr int NC = TL::kFragChunks;
  constexpr int RPI = 64 / CPR;                     // rows one copy instruction fills
  constexpr int PF = kScoreTile / RPI / kBlkWaves;  // copy instructions per wave and tile
  constexpr int kTileBytes = kScoreTile * RBt;
  constexpr int kStageBytes = blocks_stage_bytes<T, D>();
  static_assert(64 % CPR == 0 && kScoreTile % (RPI * kBlkWaves) == 0, "the copy instructions must tile a tile evenly");
  extern __shared__ __align__(16) char smem[];
  // smem: the key tile, then the two stages
  float* colacc = reinterpret_cast<float*>(smem + kTileBytes + 2 * kStageBytes);  // [Hkv][128] column sums, all row blocks
  float* colred = colacc + a.Hkv * kScoreTile;                       // [2][128] share of the second row group
  double* red = reinterpret_cast<double*>(colred + 2 * kScoreTile);  // [waves][2]

  // Tile t is seen by NT - t row blocks: the longest workgroups go first (tile 0 of all layers, then tile 1, ...).
  const int id = blockIdx.y * gridDim.x + blockIdx.x;
  const int tile = id / a.L;
  const int l = a.L - 1 - (id - tile * a.L);
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cw = wave & 3, rh = wave >> 2;
  const int j0 = tile * kScoreTile;
  const int j = j0 + cw * 32 + n;  // this lane's key column
  const bool col_is_vision = j < a.Tk && a.mask[(size_t)(l / a.Lseq) * a.Tk + j] != 0;
  const int coef_plane = col_is_vision ? 1 : 2;  // text rows weigh vision columns, vision rows text columns
  // row blocks that exist (the scoring rows are the last q_rows positions) and see this tile
  const int n_bi = min((a.Tk - j0 + kBlkRows - 1) / kBlkRows, (a.q_rows + kBlkRows - 1) / kBlkRows);
  const int n_items = n_bi * a.Hq * 2;                     // (row block, head, half), the half running fastest

  for (int i = tid; i < a.Hkv * kScoreTile; i += kBlkThreads) colacc[i] = 0.f;  // published by the first barrier

  // Copy instruction c of this wave fills the rows (wave * PF + c) * RPI .. + RPI-1 of a tile: this lane brings one
  // 16-byte chunk of the row crow + c * RPI.  Key rows past the end of the sequence repeat the last key, query and
  // statistics rows past it the last row: such columns and rows are masked below, they only have to be readable.
  const int crow = wave * PF * RPI + lane / CPR;
  unsigned koff[PF];    // byte offset of this lane's piece inside the keys of a (layer, kv head): the same for all items
  unsigned qchunk[PF];  // its chunk offset inside a query row
#pragma unroll
  for (int c = 0; c < PF; ++c) {
    const int r = crow + c * RPI;
    qchunk[c] = (unsigned)(((lane % CPR) ^ swizzle_of_row<T, D>(r)) * 16);
    koff[c] = (unsigned)min(j0 + r, a.Tk - 1) * RBt + qchunk[c];
  }
  const unsigned lds0 = (unsigned)(size_t)smem;
  const float* stats_f = reinterpret_cast<const float*>(a.stats);
  // Row block bi holds the positions [Tb - Wb, Tb), Tb = Tk - bi * 256, Wb = min(256, q_rows - bi * 256): the scoring
  // rows are the last q_rows positions, row r of the query and statistics buffers is the position Tk - q_rows + r.
  // Half hf of a block starts at the position Tb - Wb + hf * 128 (the last block may leave the second half short or
  // empty: its rows are masked).
  auto issue = [&](int item) {
    const int hf = item & 1, hh = item >> 1;
    const int bi = hh / a.Hq, h = hh - bi * a.Hq;
    const int g = h / a.G;
    const int row0 = a.q_rows - bi * kBlkRows - min(kBlkRows, a.q_rows - bi * kBlkRows) + hf * kBlkHalf;  // in the buffers
    const unsigned stage = lds0 + (unsigned)(kTileBytes + (item & 1) * kStageBytes);
    if (hf == 0 && h - g * a.G == 0) {
      // The key tile changes with the kv head.  One buffer is enough: every wave took its key fragment out of it
      // in the first half of the previous kv head, at least one barrier ago.
      const char* ksrc = uniform_ptr(a.k + (size_t)(l * a.Hkv + g) * a.Tk * RBt);
#pragma unroll
      for (int c = 0; c < PF; ++c) async_copy16_to_lds_stream(ksrc, koff[c], lds0 + (unsigned)((wave * PF + c) * 1024));
    }
    const char* qsrc = uniform_ptr(a.q + (size_t)(l * a.Hq + h) * a.q_rows * RBt);
#pragma unroll
    for (int c = 0; c < PF; ++c) {
      const unsigned goff = (unsigned)min(row0 + crow + c * RPI, a.q_rows - 1) * RBt + qchunk[c];
      async_copy16_to_lds(qsrc, goff, stage + (unsigned)((wave * PF + c) * 1024));
    }
    // wave w brings the rows (w & 1) * 64 .. + 63 of plane w >> 1 of the row statistics
    const float* ssrc = uniform_ptr(stats_f + ((size_t)(l * a.Hq + h) * 4 + (wave >> 1)) * a.stats_rows);
    const unsigned soff = (unsigned)min(row0 + (wave & 1) * 64 + lane, a.q_rows - 1) * 4u;
    async_copy4_to_lds(ssrc, soff, stage + (unsigned)(kTileBytes + ((wave >> 1) * kBlkHalf + (wave & 1) * 64) * 4));
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

  float pbar[2][2][16];  // [half][fragment of the wave][accumulator register]
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int rbl = 0; rbl < 2; ++rbl)
#pragma unroll
      for (int r = 0; r < 16; ++r) pbar[hf][rbl][r] = 0.f;
  double ent = 0.0;  // - sum of p log p over this lane's column, all row blocks
  Frag<T, D> kf;
  float colsum = 0.f;
  float pending = 0.f;  // column sum of a finished kv head, waiting for the other row group's share
  int pending_g = -1, pending_buf = 0;
  // Adds the second row group's share (left in colred before the last barrier) to the column sums.
  auto flush_pending = [&]() {
    if (pending_g >= 0 && rh == 0 && kg == 0)
      colacc[pending_g * kScoreTile + cw * 32 + n] += pending + colred[pending_buf * kScoreTile + cw * 32 + n];
    pending_g = -1;
  };

  // one half of a (row block, head) item; hf is a compile-time constant so that pbar stays in registers
  auto half_item = [&](int hh, auto hf_tag) {
    constexpr int hf = decltype(hf_tag)::value;
    const int item = hh * 2 + hf;
    async_copy_wait<0>();  // this wave's pieces of the half have landed
    __syncthreads();       // every wave's have; and nobody reads the other stage (the previous half) any more
    flush_pending();
    if (item + 1 < n_items) issue(item + 1);

    const int bi = hh / a.Hq, h = hh - bi * a.Hq;
    const int g = h / a.G, hg = h - g * a.G;
    const int Tb = a.Tk - bi * kBlkRows, Wb = min(kBlkRows, a.q_rows - bi * kBlkRows);
    const int pos0 = Tb - Wb + hf * kBlkHalf;          // position of the half's first row
    const int rows = min(kBlkHalf, Wb - hf * kBlkHalf);  // rows the half really has (may be <= 0)
    const char* stage = smem + kTileBytes + (item & 1) * kStageBytes;
    const float* st = reinterpret_cast<const float*>(stage + kTileBytes);
    if (hf == 0 && hg == 0) {
      frag_from(kf, smem + cw * 32 * RBt);  // the key tile of this kv head
      colsum = 0.f;
    }
    const bool col_ok = j < Tb;
    const bool full = rows == kBlkHalf && j0 + kScoreTile - 1 <= pos0;  // below the causal diagonal of every row
    // One query head against the wave's key columns.  MASKED: the tile touches the causal diagonal or the end of
    // the sequence, or the half is short, so every probability is checked against its row; all other tiles take
    // the plain path.
    auto head_block = [&](auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      // Row r of the half (without the lane group's offset kg*4) counts for this lane's column iff
      // row_min <= r < row_end: the row exists (r + kg*4 < rows) and sees the column (j <= pos0 + r + kg*4).
      int row_min = col_ok ? j - pos0 - kg * 4 : (1 << 30);
      int row_end = rows - kg * 4;
      if (MASKED) asm volatile("" : "+v"(row_min), "+v"(row_end));
#pragma unroll
      for (int rbl = 0; rbl < 2; ++rbl) {
        const int rb = rh * 2 + rbl;
        Frag<T, D> qf;
        frag_from(qf, stage + rb * 32 * RBt);
        // the accumulators start at the rows' biases, so that the products come out as log2 p / c
        f32x16_t acc;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 b4 = *reinterpret_cast<const float4*>(st + rb * 32 + r4 * 8 + kg * 4);
          acc[r4 * 4 + 0] = b4.x;
          acc[r4 * 4 + 1] = b4.y;
          acc[r4 * 4 + 2] = b4.z;
          acc[r4 * 4 + 3] = b4.w;
        }
        mma<T, D>(acc, qf, kf);
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int row0 = rb * 32 + r4 * 8 + kg * 4;  // rows of acc[r4*4 .. r4*4+3]
          const float4 c4 = *reinterpret_cast<const float4*>(st + coef_plane * kBlkHalf + row0);
          const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float e = fast_exp2(acc[r4 * 4 + i] * a.c);
            // rows past the block carry another row's bias and weight (finite): the select drops them
            if (MASKED) e = (rb * 32 + r4 * 8 + i >= row_min && rb * 32 + r4 * 8 + i < row_end) ? e : 0.f;
            colsum += e;
            pbar[hf][rbl][r4 * 4 + i] = fmaf(e, cc[i], pbar[hf][rbl][r4 * 4 + i]);
          }
        }
      }
    };
    if (full)
      head_block(std::false_type{});
    else
      head_block(std::true_type{});

    if (hf == 1 && hg == a.G - 1) {  // the kv head is complete for this row block
      const int buf = (bi * a.Hkv + g) & 1;  // written again two kv heads later, read after the next barrier
      const float tot = colsum + __shfl_xor(colsum, 32, kWave);
      if (rh == 1 && kg == 0) colred[buf * kScoreTile + cw * 32 + n] = tot;
      pending = tot;
      pending_g = g;
      pending_buf = buf;
    }
    if (hf == 1 && h == a.Hq - 1) {
      // entropy terms of the head-averaged cross-modal probabilities of this row block.  A vision column only
      // receives probability from text rows (text -> vision direction) and a text column only from vision rows.
      const float inv_heads = 1.0f / (float)a.Hq;
      float s = 0.f;
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int rbl = 0; rbl < 2; ++rbl)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = pbar[f][rbl][r] * inv_heads;
            s += (p > 0.f) ? p * __logf(p) : 0.f;
            pbar[f][rbl][r] = 0.f;
          }
      ent -= (double)s;
    }
  };

  issue(0);
  for (int hh = 0; hh < n_bi * a.Hq; ++hh) {
    half_item(hh, std::integral_constant<int, 0>{});
    half_item(hh, std::integral_constant<int, 1>{});
  }
  __syncthreads();
  flush_pending();
  const double tv = wave_sum(col_is_vision ? ent : 0.0);
  const double vt = wave_sum(col_is_vision ? 0.0 : ent);
  if (lane == 0) {
    red[wave * 2 + 0] = tv;
    red[wave * 2 + 1] = vt;
  }
  __syncthreads();
  for (int i = tid; i < a.Hkv * kScoreTile; i += kBlkThreads) {
    const int g = i / kScoreTile, c = i - g * kScoreTile;
    if (j0 + c < a.Tk) a.col_scores[(size_t)(l * a.Hkv + g) * a.Tk + j0 + c] = colacc[i];
  }
  if (tid < 2) {
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < kBlkWaves; ++w) sum += red[w * 2 + tid];
    a.ent_part[((size_t)l * a.NTk + tile) * 2 + tid] = sum;
  }
}

// ------------------------------------------------------------------------------------------ launch

template <typename T, int D>
static hipError_t launch_blocks_t(const Plan& p, const ScoreArgs& a, hipStream_t s) {
  const size_t lds = blocks_lds_bytes<T, D>(p.Hkv);
  auto kern = score_accum_blocks_kernel<T, D>;
  if (lds > 64 * 1024) {
    hipError_t e = allow_dynamic_lds(kern, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(p.NT, p.L), dim3(kBlkThreads), lds, s, a);
  return hipGetLastError();
}

// Rows of at most 256 bytes (two stages of 64 KB) and few enough kv heads for the column sums to fit beside them.
bool score_accum_blocks_supported(const Plan& p) {
  if (!p.blocks || p.d * p.elt > 256) return false;
  const size_t lds = p.dtype == MEDA_BF16 ? (p.d == 128 ? blocks_lds_bytes<bf16_t, 128>(p.Hkv) : blocks_lds_bytes<bf16_t, 64>(p.Hkv))
                                          : blocks_lds_bytes<float, 64>(p.Hkv);
  return lds <= 160 * 1024;
}

hipError_t launch_score_accum_blocks(const Plan& p, const Buffers& b, hipStream_t s) {
  const ScoreArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_blocks_t<bf16_t, 128>(p, a, s) : launch_blocks_t<bf16_t, 64>(p, a, s);
  return launch_blocks_t<float, 64>(p, a, s);
}

}  // namespace meda
