// C ABI of libmeda: parameter validation, workspace layout, the launch sequence of the compression
// pass, optional per-phase event timing.
#include <math.h>

#include <mutex>
#include <vector>

#include "plan.hpp"

namespace meda {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Tiling of the two scoring passes for w query rows (the last w positions) of a sequence of t keys.  With
// `single_chunk` a pass-A workgroup walks all keys its rows see (used when every prompt row scores: the row blocks
// already give that launch tens of thousands of workgroups).
static bool score_geometry(Plan* pl, int t, int w, int rows, bool single_chunk) {
  pl->Tb = t;
  pl->Wb = w;
  pl->RB = (w + 31) / 32;
  pl->Wp = pl->RB * 32;
  // Row blocks of one pass-A workgroup.  When every prompt row scores (single_chunk), pass A cuts the rows into its
  // own, larger blocks: about 16 (head, 32-row block) pairs per workgroup, so a key tile staged in LDS serves 512
  // rows without head grouping (the keys are re-read once per row block of pass A).
  pl->RBa = pl->RB;
  if (single_chunk) {
    const int want = pl->G >= 16 ? 1 : 16 / pl->G;
    const int have = (rows + 31) / 32;
    pl->RBa = want < have ? want : have;
  }
  pl->row_block_a = pl->RBa * 32;
  pl->n_blocks_a = single_chunk ? (rows + pl->row_block_a - 1) / pl->row_block_a : 1;
  const int combos = pl->G * pl->RBa;
  if (combos > 32 || pl->RB > 4) return false;
  pl->NQ = combos <= 4 ? 1 : (combos <= 16 ? 2 : 4);  // (head, row block) pairs a wave keeps in registers
  pl->NCG = (combos + pl->NQ - 1) / pl->NQ;
  pl->CS = (pl->NCG <= 4) ? 4 / pl->NCG : 1;
  const int tiles = (t + kScoreTile - 1) / kScoreTile;
  pl->NT = tiles;
  const int64_t units = (int64_t)pl->L * pl->Hkv;
  int64_t nch = single_chunk ? 1 : (4096 + units - 1) / units;
  if (nch < 1) nch = 1;
  if (nch > tiles) nch = tiles;
  const int tiles_per_chunk = (int)((tiles + nch - 1) / nch);
  pl->CH = tiles_per_chunk * kScoreTile;
  pl->NCH = (t + pl->CH - 1) / pl->CH;
  pl->NPART = pl->NCH * pl->CS;
  return true;
}

meda_status make_plan(const meda_params* p, Plan* out) {
  if (!p) return MEDA_ERR_INVALID_ARG;
  if (p->n_layers < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->seq_len < 1 || p->window < 1)
    return MEDA_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return MEDA_ERR_INVALID_ARG;
  if (p->window > p->seq_len) return MEDA_ERR_INVALID_ARG;
  if (p->recent_den <= 0 || p->recent_num < 0 || p->recent_num > p->recent_den) return MEDA_ERR_INVALID_ARG;
  if (!(p->softmax_scale >= 0.0f) || !isfinite(p->softmax_scale)) return MEDA_ERR_INVALID_ARG;
  if (p->dtype != MEDA_F32 && p->dtype != MEDA_BF16) return MEDA_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return MEDA_ERR_UNSUPPORTED;
  if (p->n_seqs < 0) return MEDA_ERR_INVALID_ARG;
  const int n_seqs = p->n_seqs > 0 ? p->n_seqs : 1;
  const int64_t layers = (int64_t)n_seqs * p->n_layers;  // layers of the whole batch
  if (layers > kMaxLayers) return MEDA_ERR_UNSUPPORTED;
  if (layers * p->n_kv_heads * (int64_t)p->seq_len >= (1ll << 31)) return MEDA_ERR_UNSUPPORTED;
  {
    // row statistics are indexed with 32 bits over [layers][Hq][scoring rows, at least one padded window of 128];
    // offsets inside one (layer, head) of q, k, v are 32-bit byte counts
    const int64_t rows = (p->flags & MEDA_FLAG_FULL_PROMPT) ? p->seq_len : p->window;
    if (layers * p->n_q_heads * (rows > 128 ? rows : 128) >= (1ll << 31)) return MEDA_ERR_UNSUPPORTED;
    const int64_t elt = (p->dtype == MEDA_BF16) ? 2 : 4;
    if ((int64_t)p->seq_len * p->head_dim * elt >= (1ll << 31)) return MEDA_ERR_UNSUPPORTED;
  }
  {
    const int64_t lo1 = (int64_t)p->n_layers * (p->window < p->seq_len ? p->window : p->seq_len);
    if (p->total_budget < lo1 || p->total_budget > (int64_t)p->n_layers * p->seq_len) return MEDA_ERR_BUDGET;
  }

  Plan pl;
  pl.N = n_seqs; pl.Lseq = p->n_layers;
  pl.L = (int)layers; pl.Hq = p->n_q_heads; pl.Hkv = p->n_kv_heads; pl.G = pl.Hq / pl.Hkv;
  pl.d = p->head_dim; pl.T = p->seq_len; pl.W = p->window; pl.B = p->total_budget * n_seqs;
  pl.num = p->recent_num; pl.den = p->recent_den; pl.dtype = p->dtype; pl.flags = p->flags;
  pl.elt = (p->dtype == MEDA_BF16) ? 2 : 4;
  const int64_t lo = (int64_t)pl.L * (pl.W < pl.T ? pl.W : pl.T), hi = (int64_t)pl.L * pl.T;
  if (pl.B < lo || pl.B > hi) return MEDA_ERR_BUDGET;
  const double scale = (p->softmax_scale > 0.0f) ? (double)p->softmax_scale : 1.0 / sqrt((double)pl.d);
  pl.scale_log2 = (float)(scale * 1.4426950408889634074);

  const bool full_prompt = (pl.flags & MEDA_FLAG_FULL_PROMPT) != 0;
  pl.R = full_prompt ? pl.T : pl.W;
  // More than 128 scoring rows (a long observation window, or every prompt row), or more (head, 32-row block) pairs
  // per kv head than a workgroup of the window kernels holds: the rows are cut into row blocks counted from the end,
  // and one launch of each scoring kernel covers all of them.
  pl.blocks = (pl.R > kScoreRowBlock || pl.G * ((pl.R + 31) / 32) > 32) ? 1 : 0;
  pl.Tk = pl.T;
  pl.q_row0 = 0;
  pl.NTk = (pl.T + kScoreTile - 1) / kScoreTile;
  pl.accumulate = 0;
  const int w_score = (pl.blocks || pl.R > kScoreRowBlock) ? kScoreRowBlock : pl.R;
  if (!score_geometry(&pl, pl.T, w_score, pl.R, pl.blocks)) return MEDA_ERR_UNSUPPORTED;
  const size_t stats_rows = pl.blocks ? (size_t)pl.R : (size_t)pl.Wp;

  pl.n_less_total = (size_t)((int64_t)pl.L * pl.T - pl.B) * pl.Hkv;
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o = align_up(o + bytes, 256); return at; };
  pl.off_stats_part = take((size_t)pl.L * pl.Hq * stats_rows * pl.NPART * 16);
  pl.off_stats = take((size_t)pl.L * pl.Hq * stats_rows * 16);
  pl.off_inv_norm = take((size_t)pl.L * pl.Hkv * pl.T * 4);
  pl.off_col_scores = take((size_t)pl.L * pl.Hkv * pl.T * 4);
  pl.off_ent_part = take((size_t)pl.L * pl.NTk * 2 * 8);
  pl.off_alloc = take((size_t)pl.L * 16);
  pl.off_layer_off = take((size_t)(pl.L + 1) * 8);
  pl.off_sel_idx = take((size_t)pl.B * pl.Hkv * 4);
  pl.off_sel_inv = take((size_t)pl.B * pl.Hkv * 4);
  pl.off_packed_k = take((size_t)pl.B * pl.Hkv * pl.d * pl.elt);
  const size_t less_bytes = pl.n_less_total * 4 + 16;
  pl.off_less_idx = take(less_bytes);
  pl.off_less_slot = take(less_bytes);
  pl.off_sort_a = take(less_bytes);
  pl.off_sort_b = take(less_bytes);
  pl.off_sort_c = take(less_bytes);
  pl.off_sort_d = take(less_bytes);
  pl.off_seg_beg = take((size_t)pl.B * pl.Hkv * 4);
  pl.off_seg_end = take((size_t)pl.B * pl.Hkv * 4);
  pl.total_bytes = o;
  *out = pl;
  return MEDA_OK;
}

// Kernels whose dynamic LDS limit has been raised, per device (a few dozen template instantiations at most).
hipError_t allow_dynamic_lds(const void* kernel, int bytes) {
  struct Entry { const void* fn; int bytes; unsigned long long devices; };
  static std::mutex mu;
  static std::vector<Entry> seen;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  std::lock_guard<std::mutex> lk(mu);
  Entry* entry = nullptr;
  for (Entry& en : seen)
    if (en.fn == kernel && en.bytes >= bytes) entry = &en;
  if (entry && tracked && ((entry->devices >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess || !tracked) return e;
  if (entry) entry->devices |= 1ull << dev;
  else seen.push_back(Entry{kernel, bytes, 1ull << dev});
  return hipSuccess;
}

// ------------------------------------------------------------------------------------- profiling
struct CallEvents {
  hipEvent_t ev[MEDA_N_PHASES + 1];
  int only;  // -1: every phase was bracketed; p: only phase p (events p and p+1)
};
static std::mutex g_mu;
static bool g_profile = false;
static int g_only = -1;
static std::vector<CallEvents> g_pending, g_pool;
static double g_ms[MEDA_N_PHASES] = {0};
static int g_calls = 0;
constexpr size_t kMaxPending = 4096;

static bool acquire_events(CallEvents* ce) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_profile || g_pending.size() >= kMaxPending) return false;
  if (!g_pool.empty()) {
    *ce = g_pool.back();
    g_pool.pop_back();
  } else {
    for (int i = 0; i <= MEDA_N_PHASES; ++i)
      if (hipEventCreate(&ce->ev[i]) != hipSuccess) return false;
  }
  ce->only = g_only;
  return true;
}

}  // namespace meda

using namespace meda;

extern "C" {

size_t meda_workspace_bytes(const meda_params* params) {
  Plan pl;
  if (make_plan(params, &pl) != MEDA_OK) return 0;
  return pl.total_bytes;
}

meda_status meda_workspace_region(const meda_params* params, int region, size_t* offset, size_t* bytes) {
  Plan pl;
  if (!offset || !bytes) return MEDA_ERR_INVALID_ARG;
  const meda_status st = make_plan(params, &pl);
  if (st != MEDA_OK) return st;
  switch (region) {
    case MEDA_REGION_COL_SCORES: *offset = pl.off_col_scores; *bytes = (size_t)pl.L * pl.Hkv * pl.T * 4; break;
    case MEDA_REGION_INV_NORM: *offset = pl.off_inv_norm; *bytes = (size_t)pl.L * pl.Hkv * pl.T * 4; break;
    case MEDA_REGION_ROW_STATS:
      *offset = pl.off_stats;
      *bytes = (size_t)pl.L * pl.Hq * (pl.blocks ? (size_t)pl.R : (size_t)pl.Wp) * 16;
      break;
    case MEDA_REGION_ALLOC: *offset = pl.off_alloc; *bytes = (size_t)pl.L * 16; break;
    case MEDA_REGION_LESS_IDX: *offset = pl.off_less_idx; *bytes = pl.n_less_total * 4; break;
    case MEDA_REGION_LESS_SLOT: *offset = pl.off_less_slot; *bytes = pl.n_less_total * 4; break;
    default: return MEDA_ERR_INVALID_ARG;
  }
  return MEDA_OK;
}

meda_status meda_compress(const meda_params* params, const void* q_win, const void* k, const void* v,
                          const uint8_t* modality, void* k_out, void* v_out, int32_t* layer_len,
                          int64_t* layer_off, double* entropy, int32_t* sel_idx, int32_t* merge_assign,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan pl;
  const meda_status st = make_plan(params, &pl);
  if (st != MEDA_OK) return st;
  if (!q_win || !k || !v || !modality || !k_out || !v_out || !layer_len || !layer_off) return MEDA_ERR_INVALID_ARG;
  if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < pl.total_bytes) return MEDA_ERR_WORKSPACE;
  const uintptr_t align_or = (uintptr_t)q_win | (uintptr_t)k | (uintptr_t)v | (uintptr_t)k_out | (uintptr_t)v_out;
  if (align_or & 15u) return MEDA_ERR_INVALID_ARG;  // rows are moved in 16-byte pieces

  Buffers b;
  b.q = q_win; b.k = k; b.v = v; b.mask = modality; b.k_out = k_out; b.v_out = v_out;
  b.layer_len = layer_len; b.layer_off = layer_off; b.entropy = entropy; b.sel_idx_user = sel_idx;
  b.merge_assign = merge_assign; b.ws = static_cast<char*>(workspace);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  CallEvents ce;
  const bool prof = acquire_events(&ce);
  typedef hipError_t (*Launcher)(const Plan&, const Buffers&, hipStream_t);
  const Launcher phases[MEDA_N_PHASES] = {launch_score_stats, launch_stats_combine, launch_score_accum,
                                          launch_allocate,    launch_select,        launch_similarity,
                                          launch_segment_sort, launch_merge_write};
  const bool no_merge = (pl.flags & MEDA_FLAG_NO_MERGE) || pl.B == (int64_t)pl.L * pl.T;
  hipError_t err = hipSuccess;
  if (prof && ce.only <= 0) err = hipEventRecord(ce.ev[0], s);
  for (int i = 0; i < MEDA_N_PHASES && err == hipSuccess; ++i) {
    const bool skip = no_merge && (i == 5 || i == 6);
    if (!skip) err = phases[i](pl, b, s);
    const bool rec = prof && (ce.only < 0 || i == ce.only || i + 1 == ce.only);
    if (rec && err == hipSuccess) err = hipEventRecord(ce.ev[i + 1], s);
  }
  if (prof) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (err == hipSuccess) g_pending.push_back(ce); else g_pool.push_back(ce);
  }
  return err == hipSuccess ? MEDA_OK : MEDA_ERR_HIP;
}

meda_status meda_profile_enable(int enable) {
  if (enable < 0 || enable > 1 + MEDA_N_PHASES) return MEDA_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_mu);
  g_profile = enable != 0;
  g_only = enable >= 2 ? enable - 2 : -1;
  return MEDA_OK;
}

meda_status meda_profile_read(double* phase_ms, int32_t* n_calls, int reset) {
  if (!phase_ms || !n_calls) return MEDA_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_mu);
  meda_status st = MEDA_OK;
  for (CallEvents& ce : g_pending) {
    const int last = ce.only < 0 ? MEDA_N_PHASES : ce.only + 1;
    if (hipEventSynchronize(ce.ev[last]) != hipSuccess) { st = MEDA_ERR_HIP; continue; }
    for (int i = 0; i < MEDA_N_PHASES; ++i) {
      if (ce.only >= 0 && i != ce.only) continue;
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ce.ev[i], ce.ev[i + 1]) == hipSuccess) g_ms[i] += ms; else st = MEDA_ERR_HIP;
    }
    ++g_calls;
    g_pool.push_back(ce);
  }
  g_pending.clear();
  for (int i = 0; i < MEDA_N_PHASES; ++i) phase_ms[i] = g_ms[i];
  *n_calls = g_calls;
  if (reset) {
    for (int i = 0; i < MEDA_N_PHASES; ++i) g_ms[i] = 0.0;
    g_calls = 0;
  }
  return st;
}

const char* meda_phase_name(int phase) {
  static const char* names[MEDA_N_PHASES] = {"score_stats", "stats_combine", "score_accum", "allocate",
                                             "select",      "similarity",    "segment_sort", "merge_write"};
  return (phase >= 0 && phase < MEDA_N_PHASES) ? names[phase] : "?";
}

const char* meda_status_string(meda_status status) {
  switch (status) {
    case MEDA_OK: return "ok";
    case MEDA_ERR_INVALID_ARG: return "invalid argument";
    case MEDA_ERR_BUDGET: return "total budget outside [L*min(W,T), L*T]";
    case MEDA_ERR_UNSUPPORTED: return "unsupported head_dim, dtype, window or group size";
    case MEDA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MEDA_ERR_HIP: return "HIP error";
    case MEDA_ERR_SCRATCH_LIMIT: return "the step needs more scratch than the no-allocation entry point's built-in array holds";
  }
  return "unknown status";
}

}  // extern "C"
