// Host-side launch plan: everything derived from meda_params (tile counts, workspace regions) and
// the entry points of the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/meda.h"

namespace meda {

constexpr int kScoreTile = 128;   // key columns per LDS tile in the two scoring passes
constexpr int kSimRowsPerWave = 64;
constexpr int kSimWaves = 4;
constexpr int kSimRows = kSimRowsPerWave * kSimWaves;  // less-important rows per workgroup
constexpr int kSimSlotTile = 64;                       // conserved slots staged in LDS per step
constexpr int kMaxLayers = 256;
constexpr int kScoreRowBlock = 128;  // query rows per row block of pass B when every prompt row scores

struct Plan {
  // problem.  A batch of N sequences is laid out as N * Lseq "layers": every kernel but the budget
  // allocation treats layers independently, so L and B below are totals over the batch and only the
  // modality mask (one per sequence: layer l uses mask + (l / Lseq) * T) and the allocation know about sequences.
  int L, Hq, Hkv, G, d, T, W;
  int N, Lseq;
  int64_t B;
  int num, den, dtype, flags;
  float scale_log2;  // softmax scale times log2(e): logits are kept in the base-2 domain
  int elt;           // bytes per element
  // scoring
  int RB, Wp;        // 32-row blocks of the window (of a 128-row block when every prompt row scores), padded window
  int RBa;           // 32-row blocks of one pass-A workgroup (RB, or more when every prompt row scores)
  int row_block_a, n_blocks_a;  // rows per row block of pass A and their number (every prompt row scores)
  int NQ, NCG, CS;   // pass A: (head, row block) pairs per wave, wave groups, column split
  int CH, NCH, NPART;  // pass A: columns per chunk, chunks, partial statistics per row
  int NT;            // pass B: column tiles
  // Scoring rows: the W window rows (R == W), or with MEDA_FLAG_FULL_PROMPT every prompt position (R == T); they are
  // the last R positions.  In the row-block mode (`blocks`: R > 128, or more (head, 32-row block) pairs per kv head
  // than the window kernels hold) the rows are cut into blocks counted from the end; a block of the positions
  // [Tb - Wb, Tb) sees only the keys below Tb, so it is the window computation of a sequence cut after its last row.
  // One launch of each scoring kernel covers all blocks (the kernels derive Tb, Wb themselves).
  int Tb, Wb;        // keys and query rows of the scoring launch (T and W; in the row-block mode: T and 128)
  int R;             // scoring rows in total; rows per (layer, head) in the query buffer
  int blocks;        // row-block mode
  int Tk;            // key rows per (layer, kv head) in memory (T of the whole sequence)
  int q_row0;        // first row of the block inside the query buffer
  int NTk;           // column tiles of the whole sequence (stride of the per-tile entropy partials)
  int accumulate;    // add to column scores / entropy partials instead of storing (every block but the first)
  // workspace regions (byte offsets)
  size_t off_stats_part, off_stats, off_inv_norm, off_col_scores, off_ent_part, off_alloc, off_layer_off,
      off_sel_idx, off_sel_inv, off_packed_k, off_less_idx, off_less_slot, off_sort_a, off_sort_b, off_sort_c, off_sort_d, off_seg_beg, off_seg_end, total_bytes;
  size_t n_less_total;  // (L*T - B) * Hkv
};

meda_status make_plan(const meda_params* p, Plan* plan);

struct Buffers {
  const void *q, *k, *v;
  const uint8_t* mask;
  void *k_out, *v_out;
  int32_t* layer_len;
  int64_t* layer_off;
  double* entropy;
  int32_t* sel_idx_user;
  int32_t* merge_assign;
  char* ws;
};

// Raises a kernel's dynamic LDS limit once per (kernel, device): the attribute is a property of the loaded
// function, and a host call per launch would sit on the critical path of the small workloads.
hipError_t allow_dynamic_lds(const void* kernel, int bytes);
template <typename K>
inline hipError_t allow_dynamic_lds(K kernel, int bytes) {
  return allow_dynamic_lds(reinterpret_cast<const void*>(kernel), bytes);
}

// kernel launchers (one per phase); each returns the hipError_t of its launch
hipError_t launch_score_stats(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_stats_combine(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_score_accum(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_allocate(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_select(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_similarity(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_segment_sort(const Plan&, const Buffers&, hipStream_t);
hipError_t launch_merge_write(const Plan&, const Buffers&, hipStream_t);

}  // namespace meda
