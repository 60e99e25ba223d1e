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
//           score_accum_dma_kernel     the same arithmetic for grouped heads, fed by asynchronous copies
//           score_accum_blocks_kernel  the row-block mode (more than 128 scoring rows)
// Logits are kept in the base-2 domain: t = (q.k) * scale * log2(e), probabilities are exp2(t - max).
// This header holds what the passes share: the argument block and its filling from the plan.  Pass A and each form
// of pass B are translation units of their own (score_stats.hip, score_accum.hip, score_accum_dma.hip,
// score_accum_blocks.hip): they sit at the edge of their register budgets and the compiler's allocation for one
// kernel shifted when another lived in the same module.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "plan.hpp"

namespace meda {

struct ScoreArgs {
  const char* q;
  const char* k;
  const uint8_t* mask;  // [N][Tk]: layer l belongs to sequence l / Lseq
  float4* stats_part;  // [L][Hq][stats_rows][NPART] (max, Z_vision, Z_text, -)
  float4* stats;       // [L][Hq][4][stats_rows] floats: planes of (max, 1/Z_all, coef for vision columns, coef for text
                       // columns), or of the form the row-block mode uses (stats_combine_kernel)
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
  // Row-block mode (blocks; q_rows scoring rows, the last positions of the sequence): the rows are cut
  // into blocks of row_block rows counted from the end; block bi holds the positions [Tb - Wb, Tb) with
  // Tb = Tk - bi * row_block, Wb = min(row_block, q_rows - bi * row_block), and sees only the keys below Tb, so it is
  // the window computation of the sequence cut at Tb.  The kernels derive T, W and q_row0 of their block themselves
  // (one launch covers all blocks).
  int blocks, row_block;
  int stats_rows;  // rows per (layer, head) in stats / stats_part (the padded window, or all q_rows rows)
  int stats_row0;  // first row of this launch's (or block's) rows in them
  float c;             // scale * log2(e)
};

// The arguments of row block bi (see ScoreArgs::blocks).
__device__ __forceinline__ void select_row_block(ScoreArgs& a, int bi) {
  a.T = a.Tk - bi * a.row_block;
  a.W = min(a.row_block, a.q_rows - bi * a.row_block);  // the first rows may leave the last block short
  a.q_row0 = a.q_rows - bi * a.row_block - a.W;
  a.stats_row0 = a.q_row0;
  a.accumulate = bi > 0;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

inline ScoreArgs make_args(const Plan& p, const Buffers& b, bool pass_a = false) {
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
  a.blocks = p.blocks; a.row_block = kScoreRowBlock;
  a.stats_rows = p.blocks ? p.R : p.Wp; a.stats_row0 = 0;
  if (pass_a) {  // pass A has its own row blocks when every prompt row scores
    a.RB = p.RBa;
    if (p.blocks) a.row_block = p.row_block_a;
  }
  a.c = p.scale_log2;
  return a;
}

// Pass B when every prompt row scores, for shapes whose items fit a two-stage LDS ring (score_accum_blocks.hip);
// the other shapes take the row-block mode of score_accum_kernel.
bool score_accum_blocks_supported(const Plan& p);
hipError_t launch_score_accum_blocks(const Plan& p, const Buffers& b, hipStream_t s);

// Pass B of the window mode for grouped heads, fed by asynchronous copies (score_accum_dma.hip); bit-identical
// results to score_accum_kernel, which keeps the other shapes.
bool score_accum_dma_supported(const Plan& p);
hipError_t launch_score_accum_dma(const Plan& p, const Buffers& b, hipStream_t s);

}  // namespace meda
