// Merging phases (Section 3.3, "Multimodal KV Pair Merging"): cosine similarity between every
// less-important key and every conserved key with a fused row argmax, a stable sort of the
// less-important positions by the slot they merge into, and the average merge of keys and values
// written straight into the ragged output.
#include "device_utils.hpp"
#include "plan.hpp"

namespace meda {

struct MergeArgs {
  const char* k;
  const char* v;
  char* k_out;
  char* v_out;
  const float* inv_norm;    // [L][Hkv][T]
  const int32_t* alloc;     // [L][4]
  const int64_t* off;       // [L+1]
  const int32_t* sel_idx;   // ragged [B*Hkv]: row id (l*Hkv+g)*T + position of every conserved key
  const float* sel_inv_norm;  // ragged: 1/|k| of the conserved keys
  const int32_t* less_idx;  // ragged: row ids of the less-important keys (ascending)
  int32_t* less_slot;       // ragged: slot each of them merges into
  int32_t* sort_key[2];     // ping-pong buffers of the segment sort
  int32_t* sort_val[2];
  int32_t* seg_beg;         // [B*Hkv]: members of output row w are sort_val[0][seg_beg[w] .. seg_end[w])
  int32_t* seg_end;
  int32_t* merge_assign;    // may be null
  int L, Hkv, T, flags;
  int merge_members;        // 0: every output row is a plain copy (no merge requested or nothing to merge)
  long long total_slots;    // B * Hkv
  int use_resident;         // layers whose conserved set fits into LDS go to the resident-set kernel
  int n_members;            // keys that are not conserved, all layers and heads: (L * T - B) * Hkv
};

__device__ __forceinline__ size_t less_base_of(int l, int g, int T, int Hkv, long long off_l, int S) {
  return ((size_t)l * T - (size_t)off_l) * Hkv + (size_t)g * (T - S);
}

// number of 5-bit passes the segment sort needs for slots in [0, S)
__device__ __forceinline__ int sort_passes(int S) {
  const int nbits = (S > 1) ? (32 - __clz(S - 1)) : 1;
  return (nbits + 4) / 5;
}

// ------------------------------------------------------------------------ similarity + argmax
// Layers whose conserved set fits into LDS go to the resident-set kernel (one workgroup of 8 waves per
// (layer, head) part, all 160 KB of LDS), the others to the tiled kernel; both are launched and every
// workgroup looks up its layer's budget.
constexpr int kResWaves = 8;
constexpr int kResThreads = kResWaves * 64;
constexpr int kResLdsBytes = 160 * 1024;
constexpr int kResSplit = 1;

// conserved keys (a multiple of 32) that fit: one padded row and one 1/|k| each
template <typename T, int D>
constexpr int resident_capacity() {
  // rows above 256 bytes would need more registers per wave than eight waves per CU leave
  return Tile<T, D>::kRowBytes > 256 ? 0 : kResLdsBytes / (Tile<T, D>::kStride + 4) / 32 * 32;
}

// grid (ceil(T / 256), Hkv, L); 4 waves x 64 less-important rows.  u_ij = (k_i . k_j)/(|k_i| |k_j|):
// the raw keys are multiplied (bf16 products are exact in the fp32 accumulator), the factor 1/|k_j|
// of the conserved key is applied to the accumulator, and the positive factor 1/|k_i| of the row is
// dropped because it cannot change the argmax over j.  Ties go to the lower slot.
//
// Each wave keeps its 64 rows as two B-operand fragments in registers for the whole kernel and
// streams the conserved keys of its (layer, head) through LDS as A operands, in tiles of 64 slots
// (double buffered: the global loads of tile t+1 and the position loads of tile t+2 are in flight
// while tile t is multiplied).  With the conserved keys as operand A, a lane owns ONE row and sees
// 16 candidate slots per 32x32 block in its 16 accumulator registers: the running best of the row is
// one value per lane and the block maximum is a max3 tree (see RowBest).
// Running best of one row (one lane) over the blocks it has seen: the best value, the first slot of
// the block that produced it and that block's 16 scaled products.  Keeping the products postpones the
// search for the winning register to the end of the kernel: per block only the maximum is formed
// (max3 tree), and the 16 products are copied in blocks where some lane of the wave improved.
struct RowBest {
  float best;
  int slot0;
  float u[16];
};

__device__ __forceinline__ void argmax_block(const f32x16_t& acc, const float (&iv)[16], int slot0, RowBest& rb) {
  float u[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) u[r] = acc[r] * iv[r];
  float bm = fmaxf(fmaxf(u[0], u[1]), u[2]);
#pragma unroll
  for (int r = 3; r < 15; r += 2) bm = fmaxf(fmaxf(bm, u[r]), u[r + 1]);
  bm = fmaxf(bm, u[15]);
  const bool improved = bm > rb.best;  // strict: an equal value in a later block does not replace
  if (__ballot(improved) != 0ull) {
#pragma unroll
    for (int r = 0; r < 16; ++r) rb.u[r] = improved ? u[r] : rb.u[r];
    rb.best = improved ? bm : rb.best;
    rb.slot0 = improved ? slot0 : rb.slot0;
  }
}

// Slot of the row's best: the lowest register of the saved block that holds the maximum.
// best - u[r] is +0 exactly there and positive elsewhere, and the bit patterns of non-negative floats
// order like unsigned integers, so the minimum of (bits << 4 | r) carries r of the first maximum.
__device__ __forceinline__ int row_best_slot(const RowBest& rb, int kg) {
  unsigned key = 0xffffffffu;
#pragma unroll
  for (int r = 0; r < 16; ++r) key = min(key, (__float_as_uint(rb.best - rb.u[r]) << 4) | (unsigned)r);
  const int ridx = (int)(key & 15u);
  return rb.slot0 + (ridx >> 2) * 8 + kg * 4 + (ridx & 3);
}

// One LDS tile of conserved keys against the wave's two row fragments.  The last tile of a (layer,
// head) is padded with copies of the last conserved key: a copy ties with the original and the tie
// rules (strict improvement, lowest register, lower slot between the lane groups) always prefer the
// original, so no slot needs masking and there is a single code path.
template <typename T, int D>
__device__ __forceinline__ void sim_tile(const char* ctile, const float* cinv, int s0, int n, int kg,
                                         const Frag<T, D> (&lf)[2], RowBest (&rb)[2]) {
  using TL = Tile<T, D>;
#pragma unroll
  for (int cb = 0; cb < kSimSlotTile / 32; ++cb) {
    Frag<T, D> cf;
    frag_load(cf, ctile + (cb * 32 + n) * TL::kStride, kg);
    float iv[16];
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const float4 v = *reinterpret_cast<const float4*>(cinv + cb * 32 + r4 * 8 + kg * 4);
      iv[r4 * 4 + 0] = v.x;
      iv[r4 * 4 + 1] = v.y;
      iv[r4 * 4 + 2] = v.z;
      iv[r4 * 4 + 3] = v.w;
    }
    f32x16_t acc0 = acc_zero(), acc1 = acc_zero();
    mma<T, D>(acc0, cf, lf[0]);
    mma<T, D>(acc1, cf, lf[1]);
    argmax_block(acc0, iv, s0 + cb * 32, rb[0]);
    argmax_block(acc1, iv, s0 + cb * 32, rb[1]);
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(kSimWaves * 64, (Tile<T, D>::kRowBytes <= 256 ? 2 : 1)) similarity_argmax_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  constexpr int CPR = TL::kChunksPerRow;
  constexpr int NTHR = kSimWaves * 64;
  constexpr int PF = kSimSlotTile * CPR / NTHR;  // 16-byte pieces of a tile per thread
  constexpr int ROWS_PER_PIECE_STEP = NTHR / CPR;
  static_assert(kSimSlotTile * CPR % NTHR == 0 && NTHR % CPR == 0, "tile pieces must divide evenly over the threads");
  __shared__ __align__(16) char ctile[2][kSimSlotTile * TL::kStride];
  __shared__ __align__(16) float cinv[2][kSimSlotTile];

  // Workgroups are dealt round-robin to the 8 XCDs in launch order.  The launch index is remapped so
  // that all row blocks of one (layer, head) run on the same XCD (they stream the same conserved keys
  // and then share one L2), while consecutive (layer, head) pairs go to different XCDs.
  const unsigned nrb = (a.T + kSimRows - 1) / kSimRows;
  const unsigned xcd = blockIdx.x & 7u, seq = blockIdx.x >> 3;
  const unsigned pair = xcd + 8u * (seq / nrb);
  if (pair >= (unsigned)(a.L * a.Hkv)) return;
  const int l = a.alloc[4 * (pair / a.Hkv) + 3], g = pair % a.Hkv;  // layers by decreasing budget
  const int S = a.alloc[4 * l];
  if (a.use_resident && S <= resident_capacity<T, D>()) return;  // the resident-set kernel below takes this layer
  const int n_less = a.T - S;
  const int row_base = (seq % nrb) * kSimRows;
  if (row_base >= n_less) return;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const long long off_l = a.off[l];
  const size_t cbase = (size_t)off_l * a.Hkv + (size_t)g * S;
  const int32_t* cidx = a.sel_idx + cbase;
  const float* sinv = a.sel_inv_norm + cbase;
  const size_t lbase = less_base_of(l, g, a.T, a.Hkv, off_l, S);
  const int32_t* less = a.less_idx + lbase;
  const char* kbase = a.k;  // positions are stored as row ids over all layers and heads

  // first the row ids this wave needs (its own rows; rows past the end repeat the last one and are
  // never stored), so that all index loads of the prologue are in flight before any row load
  const int r0 = row_base + wave * kSimRowsPerWave;
  int lrow[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) lrow[s] = less[min(r0 + s * 32 + n, n_less - 1)];
  RowBest rb[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    rb[s].best = -INFINITY;
    rb[s].slot0 = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) rb[s].u[r] = -INFINITY;
  }

  // this thread's pieces of a tile: piece i is 16 bytes at row prow0 + i * ROWS_PER_PIECE_STEP, column pcc
  const int prow0 = tid / CPR, pcc = tid - prow0 * CPR;
  int pidx[PF];
  uint4 pre[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) pre[i] = make_uint4(0, 0, 0, 0);
  float piv = 0.f;
  const int ntiles = (S + kSimSlotTile - 1) / kSimSlotTile;

#define MEDA_SIM_LOAD_IDX(t)                                                      \
  _Pragma("unroll") for (int i = 0; i < PF; ++i) {                                \
    const int slot = (t) * kSimSlotTile + prow0 + i * ROWS_PER_PIECE_STEP;        \
    pidx[i] = cidx[min(slot, S - 1)];                                             \
  }
#define MEDA_SIM_ISSUE(t)                                                                                \
  _Pragma("unroll") for (int i = 0; i < PF; ++i) {                                                       \
    pre[i] = *reinterpret_cast<const uint4*>(kbase + (size_t)pidx[i] * TL::kRowBytes + pcc * 16);        \
  }                                                                                                      \
  if (tid < kSimSlotTile) piv = sinv[min((t) * kSimSlotTile + tid, S - 1)];
#define MEDA_SIM_COMMIT(buf)                                                                             \
  _Pragma("unroll") for (int i = 0; i < PF; ++i)                                                         \
    *reinterpret_cast<uint4*>(ctile[buf] + (prow0 + i * ROWS_PER_PIECE_STEP) * TL::kStride + pcc * 16) = pre[i]; \
  if (tid < kSimSlotTile) cinv[buf][tid] = piv;

  MEDA_SIM_LOAD_IDX(0)
  Frag<T, D> lf[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) frag_load(lf[s], kbase + (size_t)lrow[s] * TL::kRowBytes, kg);
  MEDA_SIM_ISSUE(0)
  if (ntiles > 1) { MEDA_SIM_LOAD_IDX(1) }
  MEDA_SIM_COMMIT(0)
  for (int t = 0; t < ntiles; ++t) {
    __syncthreads();  // tile t is in LDS; the other buffer is no longer read
    if (t + 1 < ntiles) {
      MEDA_SIM_ISSUE(t + 1)
      if (t + 2 < ntiles) { MEDA_SIM_LOAD_IDX(t + 2) }
    }
    sim_tile<T, D>(ctile[t & 1], cinv[t & 1], t * kSimSlotTile, n, kg, lf, rb);
    if (t + 1 < ntiles) { MEDA_SIM_COMMIT((t + 1) & 1) }
  }
#undef MEDA_SIM_LOAD_IDX
#undef MEDA_SIM_ISSUE
#undef MEDA_SIM_COMMIT

  // the two lane groups saw disjoint slots of the same row: keep the better, ties -> lower slot
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int mine = row_best_slot(rb[s], kg);
    const float ov = __shfl_xor(rb[s].best, 32, kWave);
    const int oi = __shfl_xor(mine, 32, kWave);
    const bool take = ov > rb[s].best || (ov == rb[s].best && oi < mine);
    const int bi = take ? oi : mine;
    const int ri = r0 + s * 32 + n;
    if (kg == 0 && ri < n_less) {
      a.less_slot[lbase + ri] = bi;
      if (a.merge_assign) a.merge_assign[less[ri]] = bi;
    }
  }
}

// Variant for layers whose conserved set fits into LDS: one workgroup keeps ALL conserved keys of its
// (layer, head) resident and every wave streams chunks of 64 less-important rows through registers.
// After the prologue there is no barrier: the waves run independently, each MFMA phase of one wave
// overlaps the argmax phase and the row loads of the others, and the keys are read from HBM once.
// grid (kResSplit * L * Hkv): part p of a pair takes the chunks p*8 + wave, then steps of 8*kResSplit.
// Layers above the capacity are left to the tiled kernel above (and skipped there when they fit).
template <typename T, int D>
__global__ void __launch_bounds__(kResThreads, 2) similarity_resident_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  constexpr int CPR = TL::kChunksPerRow;
  extern __shared__ __align__(16) char smem[];

  // workgroups are launched in the order of decreasing budget (longest first: the last ones to start
  // are the shortest), alloc[4 * rank + 3] is the layer of that rank
  const int pair = blockIdx.x / kResSplit, part = blockIdx.x % kResSplit;
  const int l = a.alloc[4 * (pair / a.Hkv) + 3], g = pair % a.Hkv;
  const int S = a.alloc[4 * l];
  const int n_less = a.T - S;
  if (S > resident_capacity<T, D>() || n_less == 0) return;
  const int n_chunks = (n_less + kSimRowsPerWave - 1) / kSimRowsPerWave;
  if (part * kResWaves >= n_chunks) return;

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long off_l = a.off[l];
  const size_t cbase = (size_t)off_l * a.Hkv + (size_t)g * S;
  const int32_t* cidx = a.sel_idx + cbase;
  const float* sinv = a.sel_inv_norm + cbase;
  const size_t lbase = less_base_of(l, g, a.T, a.Hkv, off_l, S);
  const int32_t* less = a.less_idx + lbase;
  const char* kbase = a.k;  // positions are stored as row ids over all layers and heads

  // the wave's first rows are requested before the conserved set, so they arrive during the prologue
  int c = part * kResWaves + wave;
  constexpr int kChunkStep = kResWaves * kResSplit;
  auto chunk_rows = [&](int chunk, int (&rows)[2]) {
#pragma unroll
    for (int s = 0; s < 2; ++s) rows[s] = less[min(chunk * kSimRowsPerWave + s * 32 + n, n_less - 1)];
  };
  int lrow[2], nrow[2];
  chunk_rows(c, lrow);
  chunk_rows(c + kChunkStep, nrow);
  Frag<T, D> lf[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) frag_load(lf[s], kbase + (size_t)lrow[s] * TL::kRowBytes, kg);

  // Prologue: gather the conserved keys into LDS.  The set is padded to a multiple of 32 slots with
  // copies of the last key (a copy can never win a tie against the original, see sim_tile).
  const int S_pad = (S + 31) & ~31;
  char* ckeys = smem;
  float* cinv = reinterpret_cast<float*>(smem + (size_t)S_pad * TL::kStride);
  constexpr int kBatch = 6;  // pieces per thread whose loads are in flight together
  const int n_pieces = S_pad * CPR;
  for (int p0 = tid; p0 < n_pieces; p0 += kBatch * kResThreads) {
    int ridx[kBatch];
    uint4 v[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int p = min(p0 + i * kResThreads, n_pieces - 1);
      ridx[i] = cidx[min(p / CPR, S - 1)];
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int p = min(p0 + i * kResThreads, n_pieces - 1);
      v[i] = *reinterpret_cast<const uint4*>(kbase + (size_t)ridx[i] * TL::kRowBytes + (p % CPR) * 16);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int p = p0 + i * kResThreads;
      if (p < n_pieces) *reinterpret_cast<uint4*>(ckeys + (p / CPR) * TL::kStride + (p % CPR) * 16) = v[i];
    }
  }
  for (int sl = tid; sl < S_pad; sl += kResThreads) cinv[sl] = sinv[min(sl, S - 1)];
  __syncthreads();

  while (c < n_chunks) {
    // the rows of the wave's next chunk and the row ids of the one after it are in flight while
    // this chunk is multiplied (past the last chunk they repeat the last row and are dropped)
    const int r0 = c * kSimRowsPerWave;
    Frag<T, D> lfn[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) frag_load(lfn[s], kbase + (size_t)nrow[s] * TL::kRowBytes, kg);
    int nnrow[2];
    chunk_rows(c + 2 * kChunkStep, nnrow);
    RowBest rb[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      rb[s].best = -INFINITY;
      rb[s].slot0 = 0;
#pragma unroll
      for (int r = 0; r < 16; ++r) rb[s].u[r] = -INFINITY;
    }
    for (int s0 = 0; s0 < S_pad; s0 += 32) {
      Frag<T, D> cf;
      frag_load(cf, ckeys + (s0 + n) * TL::kStride, kg);
      float iv[16];
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const float4 v = *reinterpret_cast<const float4*>(cinv + s0 + r4 * 8 + kg * 4);
        iv[r4 * 4 + 0] = v.x;
        iv[r4 * 4 + 1] = v.y;
        iv[r4 * 4 + 2] = v.z;
        iv[r4 * 4 + 3] = v.w;
      }
      f32x16_t acc0 = acc_zero(), acc1 = acc_zero();
      mma<T, D>(acc0, cf, lf[0]);
      mma<T, D>(acc1, cf, lf[1]);
      argmax_block(acc0, iv, s0, rb[0]);
      argmax_block(acc1, iv, s0, rb[1]);
    }
    // the two lane groups saw disjoint slots of the same row: keep the better, ties -> lower slot
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int mine = row_best_slot(rb[s], kg);
      const float ov = __shfl_xor(rb[s].best, 32, kWave);
      const int oi = __shfl_xor(mine, 32, kWave);
      const bool take = ov > rb[s].best || (ov == rb[s].best && oi < mine);
      const int bi = take ? oi : mine;
      const int ri = r0 + s * 32 + n;
      if (kg == 0 && ri < n_less) {
        a.less_slot[lbase + ri] = bi;
        if (a.merge_assign) a.merge_assign[lrow[s]] = bi;
      }
    }
    c += kChunkStep;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      lrow[s] = nrow[s];
      nrow[s] = nnrow[s];
      lf[s] = lfn[s];
    }
  }
}

// ------------------------------------------------------------------------------- segment sort
// grid (Hkv, L).  Stable least-significant-digit radix sort (5 bits per pass) of the pairs
// (slot, row id) of one (layer, head) by slot; row ids enter ascending, so every slot's members come
// out ascending and the merge adds them in one fixed order.  The last pass always writes buffer 0.
// Per tile of blockDim elements: a lane finds the lanes of its wave with the same digit (one ballot
// per digit bit) and its rank among them, the per-wave digit counts go to LDS, wave 0 turns them into exclusive prefixes over the
// waves (and advances the running digit bases), and every element is written to its final place.
// Then seg_beg / seg_end of every slot = its range in the sorted array.
constexpr int kSortMaxThreads = 1024;
constexpr int kSortMaxWaves = kSortMaxThreads / 64;
constexpr int kSortBits = 5;
constexpr int kSortDigits = 1 << kSortBits;
constexpr int kSortItems = 4;  // tiles whose loads are issued together

// Lanes of the wave whose 5-bit digit equals this lane's (invalid lanes match nobody): one ballot per
// digit bit, each lane keeps the side of the ballot it is on.
__device__ __forceinline__ unsigned long long digit_peers(int dgt, bool valid) {
  unsigned long long peers = __ballot(valid);
#pragma unroll
  for (int b = 0; b < kSortBits; ++b) {
    const unsigned long long set = __ballot((dgt >> b) & 1);
    peers &= ((dgt >> b) & 1) ? set : ~set;
  }
  return valid ? peers : 0ull;
}

__global__ void __launch_bounds__(kSortMaxThreads, 8) segment_sort_kernel(MergeArgs a) {
  __shared__ int base[2][kSortDigits];
  __shared__ int wcnt[2][kSortMaxWaves][kSortDigits];

  const int g = blockIdx.x, l = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nthr = blockDim.x, nwaves = nthr >> 6;
  const int S = a.alloc[4 * l];
  const int n = a.T - S;
  const long long off_l = a.off[l];
  const size_t lbase = less_base_of(l, g, a.T, a.Hkv, off_l, S);
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  const int passes = sort_passes(S);

  const int32_t* in_key = a.less_slot + lbase;
  const int32_t* in_val = a.less_idx + lbase;
  for (int p = 0; p < passes; ++p) {
    const int ob = (passes - 1 - p) & 1;
    int32_t* out_key = a.sort_key[ob] + lbase;
    int32_t* out_val = a.sort_val[ob] + lbase;
    const int shift = kSortBits * p;
    if (tid < kSortDigits) base[0][tid] = 0;
    __syncthreads();
    // digit histogram: lane q of every wave counts digit q.  Four tiles are loaded at a time so
    // that their loads are in flight together.
    for (int t0 = 0; t0 < n; t0 += kSortItems * nthr) {
      int keys[kSortItems];
#pragma unroll
      for (int j = 0; j < kSortItems; ++j) {
        const int i = t0 + j * nthr + tid;
        keys[j] = (i < n) ? in_key[i] : -1;
      }
#pragma unroll
      for (int j = 0; j < kSortItems; ++j) {
        if (t0 + j * nthr < n) {
          const bool valid = keys[j] >= 0;
          const int dgt = (keys[j] >> shift) & (kSortDigits - 1);
          const unsigned long long peers = digit_peers(dgt, valid);
          if (valid && (peers & lt_mask) == 0ull) atomicAdd(&base[0][dgt], __popcll(peers));  // group leader
        }
      }
    }
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the 32 digit totals
      const int c = (lane < kSortDigits) ? base[0][lane] : 0;
      int inc = c;
#pragma unroll
      for (int o = 1; o < kSortDigits; o <<= 1) {
        const int t = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += t;
      }
      if (lane < kSortDigits) base[0][lane] = inc - c;
    }
    __syncthreads();
    // stable scatter, blockDim elements at a time in input order (loads of four tiles in flight)
    int it = 0;
    for (int s0 = 0; s0 < n; s0 += kSortItems * nthr) {
      int keys[kSortItems], vals[kSortItems];
#pragma unroll
      for (int j = 0; j < kSortItems; ++j) {
        const int i = s0 + j * nthr + tid;
        keys[j] = (i < n) ? in_key[i] : -1;
        vals[j] = (i < n) ? in_val[i] : 0;
      }
#pragma unroll
      for (int j = 0; j < kSortItems; ++j) {
        if (s0 + j * nthr < n) {
          const int cur = it & 1;
          ++it;
          const int key = keys[j], val = vals[j];
          const bool valid = key >= 0;
          const int dgt = (key >> shift) & (kSortDigits - 1);
          const unsigned long long peers = digit_peers(dgt, valid);
          const int my_rank = __popcll(peers & lt_mask);
          if (lane < kSortDigits) wcnt[cur][wave][lane] = 0;
          if (valid && my_rank == 0) wcnt[cur][wave][dgt] = __popcll(peers);  // after the zeroing: same wave, in order
          __syncthreads();
          if (wave == 0) {
            // lane (q, half): digit q = lane / 2, waves half*8 .. half*8+7; exclusive prefix over the waves
            const int q = lane >> 1, w0 = (lane & 1) * (kSortMaxWaves / 2);
            int run = 0, c[kSortMaxWaves / 2];
#pragma unroll
            for (int w2 = 0; w2 < kSortMaxWaves / 2; ++w2) {
              c[w2] = (w0 + w2 < nwaves) ? wcnt[cur][w0 + w2][q] : 0;
              run += c[w2];
            }
            const int other = __shfl_xor(run, 1, kWave);
            int pre = (lane & 1) ? other : 0;  // counts of the lower half of the waves
#pragma unroll
            for (int w2 = 0; w2 < kSortMaxWaves / 2; ++w2) {
              if (w0 + w2 < nwaves) wcnt[cur][w0 + w2][q] = pre;
              pre += c[w2];
            }
            if ((lane & 1) == 0) base[cur ^ 1][q] = base[cur][q] + run + other;
          }
          __syncthreads();
          if (valid) {
            const int pos = base[cur][dgt] + wcnt[cur][wave][dgt] + my_rank;
            out_key[pos] = key;
            out_val[pos] = val;
          }
        }
      }
    }
    __syncthreads();
    in_key = out_key;
    in_val = out_val;
  }

  // member range of every slot, as absolute indices into the sorted array
  const size_t cbase = (size_t)off_l * a.Hkv + (size_t)g * S;
  int32_t* beg = a.seg_beg + cbase;
  int32_t* end = a.seg_end + cbase;
  const int ib = (int)lbase;
  for (int i = tid; i < n; i += nthr) {
    const int kcur = in_key[i];
    const int kprev = (i > 0) ? in_key[i - 1] : -1;
    for (int s = kprev + 1; s <= kcur; ++s) beg[s] = ib + i;
    for (int s = max(kprev, 0); s < kcur; ++s) end[s] = ib + i;
  }
  const int klast = (n > 0) ? in_key[n - 1] : -1;
  for (int s = klast + 1 + tid; s < S; s += nthr) beg[s] = ib + n;
  for (int s = max(klast, 0) + tid; s < S; s += nthr) end[s] = ib + n;
}

// ------------------------------------------------------------------------------ merge + write
// A wave produces a run of consecutive output rows (layer, head, slot), one after the other.
// k_j <- (k_j + sum_{i in N_j} k_i) / (|N_j| + 1) and the same for the values (Section 3.3, average
// merging).  A lane owns one 16-byte piece of a row, so 64 lanes read 1024 bytes = several rows per
// load; sums are kept in fp64 (exact for the value ranges of a KV cache, hence independent of the
// summation order) and rounded once to the storage type.
// sum / n for a positive integer n given rinv = fl(1/n): one multiply and one exact-remainder
// correction.  When sum / n is representable the result is exactly that value, so ties of the final
// rounding to the storage type fall the same way as with a true division.
__device__ __forceinline__ double div_by_count(double sum, double n, double rinv) {
  const double q0 = sum * rinv;
  const double rem = fma(-q0, n, sum);
  return fma(rem, rinv, q0);
}

// x + y exchanged between two lane groups O lanes apart: the lower group ends with its own x plus
// the partner's x, the upper group with its own y plus the partner's y.
template <int O>
__device__ __forceinline__ double exchange_add(double x, double y, bool upper) {
  if constexpr (O == 16 || O == 32) {
    unsigned xl = (unsigned)__double2loint(x), xh = (unsigned)__double2hiint(x);
    unsigned yl = (unsigned)__double2loint(y), yh = (unsigned)__double2hiint(y);
    if constexpr (O == 32) {
      const auto lo = __builtin_amdgcn_permlane32_swap(xl, yl, false, false);
      const auto hi = __builtin_amdgcn_permlane32_swap(xh, yh, false, false);
      xl = lo[0]; yl = lo[1]; xh = hi[0]; yh = hi[1];
    } else {
      const auto lo = __builtin_amdgcn_permlane16_swap(xl, yl, false, false);
      const auto hi = __builtin_amdgcn_permlane16_swap(xh, yh, false, false);
      xl = lo[0]; yl = lo[1]; xh = hi[0]; yh = hi[1];
    }
    return __hiloint2double((int)xh, (int)xl) + __hiloint2double((int)yh, (int)yl);
  } else {
    const double send = upper ? x : y, keep = upper ? y : x;
    return keep + __shfl_xor(send, O, kWave);
  }
}

// One halving step of the reduce-scatter over lane groups O lanes apart; returns the element offset
// this lane moves to (LEN for the upper group).
template <int LEN, int O, int E>
__device__ __forceinline__ int reduce_scatter_step(double (&ak)[E], double (&av)[E], bool upper) {
#pragma unroll
  for (int i = 0; i < LEN; ++i) {
    ak[i] = exchange_add<O>(ak[i], ak[i + LEN], upper);
    av[i] = exchange_add<O>(av[i], av[i + LEN], upper);
  }
  return upper ? LEN : 0;
}

template <typename T>
struct OutConv;
template <>
struct OutConv<bf16_t> {
  static constexpr int kElems = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, double* out) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = (double)__uint_as_float(w[i] << 16);
      out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
  // store N consecutive elements sum[i] / denom, rounded once to bf16
  template <int N>
  static __device__ __forceinline__ void store(char* dst, const double* sum, double denom, double rinv) {
    if constexpr (N == 1) {
      *reinterpret_cast<uint16_t*>(dst) = (uint16_t)double_to_bf16_bits(div_by_count(sum[0], denom, rinv));
    } else {
#pragma unroll
      for (int i = 0; i < N / 2; ++i) {
        const uint32_t wv = double_to_bf16_bits(div_by_count(sum[2 * i], denom, rinv)) |
                            (double_to_bf16_bits(div_by_count(sum[2 * i + 1], denom, rinv)) << 16);
        __builtin_nontemporal_store(wv, reinterpret_cast<uint32_t*>(dst) + i);
      }
    }
  }
};
template <>
struct OutConv<float> {
  static constexpr int kElems = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, double* out) {
    out[0] = (double)__uint_as_float(v.x);
    out[1] = (double)__uint_as_float(v.y);
    out[2] = (double)__uint_as_float(v.z);
    out[3] = (double)__uint_as_float(v.w);
  }
  template <int N>
  static __device__ __forceinline__ void store(char* dst, const double* sum, double denom, double rinv) {
#pragma unroll
    for (int i = 0; i < N; ++i)
      __builtin_nontemporal_store(__double2float_rn(div_by_count(sum[i], denom, rinv)), reinterpret_cast<float*>(dst) + i);
  }
};

// Output rows one wave walks; a lane of the wave holds the list range of one of them.
constexpr int kMergeRowsPerWave = 16;

// Where a wave is in the flat sequence of load steps of its output rows: row r of the wave, element t
// of that row's list (element 0 is the conserved row itself, the others its members), and the row's
// conserved row id, first member index and list length.  All fields are uniform over the wave.
struct MergeCursor {
  int r, t, sel, beg, cnt;
};

template <typename T, int D>
__global__ void __launch_bounds__(256) merge_write_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  using CV = OutConv<T>;
  constexpr int LPR = TL::kChunksPerRow;  // lanes per row
  constexpr int MS = 64 / LPR;            // rows per load
  constexpr int STEP = 2 * MS;            // rows per step (two loads per lane and tensor)
  constexpr int E = CV::kElems;
  constexpr int R = kMergeRowsPerWave;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // output rows are walked from the last layer to the first: the similarity kernel before this one
  // touched the last layers' keys last
  const long long w_hi = a.total_slots - ((long long)blockIdx.x * 4 + wave) * R;
  if (w_hi <= 0) return;
  const long long w_lo = w_hi > R ? w_hi - R : 0;
  const int n_out = (int)(w_hi - w_lo);
  // everything a row needs is indexed by its output row w: no layer / head lookup.  Lane i keeps the
  // entry of row w_lo + i; lanes past the wave's rows keep a list of length 1 that is never loaded.
  int m_sel = 0, m_beg = 0, m_cnt = 1;
  if (lane < n_out) {
    m_sel = a.sel_idx[w_lo + lane];
    m_beg = a.seg_beg[w_lo + lane];
    m_cnt = a.seg_end[w_lo + lane] - m_beg + 1;
  }
  const int32_t* members = a.sort_val[0];
  const int sub = lane / LPR, cc = lane - sub * LPR;
  const char* kb = a.k + cc * 16;
  const char* vb = a.v + cc * 16;

  auto read_entry = [&](MergeCursor& c) {
    c.sel = __builtin_amdgcn_readlane(m_sel, c.r);
    c.beg = __builtin_amdgcn_readlane(m_beg, c.r);
    c.cnt = __builtin_amdgcn_readlane(m_cnt, c.r);
  };
  auto advance = [&](MergeCursor& c) {
    c.t += STEP;
    if (c.t >= c.cnt) {
      c.r += 1;  // at most two steps past n_out <= 16, so always a lane of the wave
      c.t = 0;
      read_entry(c);
    }
  };
  // Row ids of the two rows this lane loads in the step at c.  Every load of the loop is issued
  // unconditionally (the number of loads in flight is then the same on every path, so a wait for
  // the oldest ones leaves the younger ones in flight): list positions past the end of the row's
  // list are clamped into the list array, and their lanes load the conserved row again, which the
  // sum then skips.
  const int last_member = a.n_members - 1;
  auto step_ids = [&](const MergeCursor& c, int& i0, int& i1) {
    const int e0 = c.t + sub, e1 = e0 + MS;
    const int p0 = min(max(c.beg - 1 + e0, 0), last_member), p1 = min(c.beg - 1 + e1, last_member);
    const int m0 = members[p0], m1 = members[p1];
    i0 = (e0 != 0 && e0 < c.cnt) ? m0 : c.sel;
    i1 = (e1 < c.cnt) ? m1 : c.sel;
  };
  auto fetch = [&](int i0, int i1, uint4 (&k)[2], uint4 (&v)[2]) {
    k[0] = load16_stream(kb + (size_t)i0 * TL::kRowBytes);
    v[0] = load16_stream(vb + (size_t)i0 * TL::kRowBytes);
    k[1] = load16_stream(kb + (size_t)i1 * TL::kRowBytes);
    v[1] = load16_stream(vb + (size_t)i1 * TL::kRowBytes);
  };

  double ak[E], av[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    ak[i] = 0.0;
    av[i] = 0.0;
  }
  // sums the rows of the step at c (already loaded into k, v); finishes the output row on its last step
  auto consume = [&](const MergeCursor& c, const uint4 (&k)[2], const uint4 (&v)[2]) {
    // One unconditional use of everything the step loaded: the wait for these loads then sits here on
    // every path, instead of inside the branches below (which would leave them formally in flight on
    // the other paths and force wider waits later).
    asm volatile("" ::"v"(k[0].x), "v"(k[0].y), "v"(k[0].z), "v"(k[0].w), "v"(k[1].x), "v"(k[1].y), "v"(k[1].z),
                 "v"(k[1].w), "v"(v[0].x), "v"(v[0].y), "v"(v[0].z), "v"(v[0].w), "v"(v[1].x), "v"(v[1].y),
                 "v"(v[1].z), "v"(v[1].w));
    const long long w = w_lo + c.r;
    if (c.cnt == 1) {  // nothing merges into this row: bit-exact copy
      if (sub == 0) {
        // the output is not read again by this pass: streaming stores (measured 2-4 % on the kernel)
        store16_stream(a.k_out + (size_t)w * TL::kRowBytes + cc * 16, k[0]);
        store16_stream(a.v_out + (size_t)w * TL::kRowBytes + cc * 16, v[0]);
      }
      return;
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (c.t + u * MS + sub < c.cnt) {  // lanes past the end of the list hold a row that does not count
        double tk[E], tv[E];
        CV::unpack(k[u], tk);
        CV::unpack(v[u], tv);
#pragma unroll
        for (int i = 0; i < E; ++i) {
          ak[i] += tk[i];
          av[i] += tv[i];
        }
      }
    }
    if (c.t + STEP < c.cnt) return;
    // Last step of the row: reduce over the lane groups that read different rows.  Each exchange
    // halves the elements a lane is responsible for (the lower group keeps the lower half), so after
    // log2(MS) steps a lane holds E / MS finished sums starting at element `ebase` of its 16-byte
    // piece: the divisions and the stores are spread over all 64 lanes.
    int ebase = 0;
    if constexpr (MS >= 2) ebase += reduce_scatter_step<E / 2, LPR>(ak, av, (sub & 1) != 0);
    if constexpr (MS >= 4) ebase += reduce_scatter_step<E / 4, 2 * LPR>(ak, av, (sub & 2) != 0);
    if constexpr (MS >= 8) ebase += reduce_scatter_step<E / 8, 4 * LPR>(ak, av, (sub & 4) != 0);
    constexpr int EPL = E / MS;  // finished elements per lane
    static_assert(EPL >= 1, "a lane must end up with at least one element");
    const double denom = (double)c.cnt;
    const double rinv = 1.0 / denom;
    char* ko = a.k_out + (size_t)w * TL::kRowBytes + cc * 16 + ebase * (int)sizeof(T);
    char* vo = a.v_out + (size_t)w * TL::kRowBytes + cc * 16 + ebase * (int)sizeof(T);
    CV::template store<EPL>(ko, ak, denom, rinv);
    CV::template store<EPL>(vo, av, denom, rinv);
#pragma unroll
    for (int i = 0; i < E; ++i) {
      ak[i] = 0.0;
      av[i] = 0.0;
    }
  };

  // Three steps are in progress at any time: the rows of step n are summed while the row loads of
  // step n + 1 and the list loads of step n + 2 are in flight.  The list loads are issued before the
  // row loads, so waiting for them one round later does not wait for the younger row loads.  The
  // loop body is written out twice with the two register sets exchanged, so no loaded value is
  // copied (a copy would have to wait for its load).  Past the wave's last row the cursors point at
  // lanes that hold (row 0, empty list): those loads are harmless and never consumed.
  MergeCursor c0{0, 0, 0, 0, 1};
  read_entry(c0);
  MergeCursor c1 = c0;
  advance(c1);
  MergeCursor c2 = c1;
  advance(c2);
  int ida0, ida1, idb0, idb1;
  uint4 ka[2], va[2], kb2[2], vb2[2];
  step_ids(c0, ida0, ida1);
  step_ids(c1, idb0, idb1);
  fetch(ida0, ida1, kb2, vb2);
  // one step: true when the wave's last row is done
  auto round = [&](int& new0, int& new1, int old0, int old1, uint4 (&nk)[2], uint4 (&nv)[2], const uint4 (&ok)[2],
                   const uint4 (&ov)[2]) {
    step_ids(c2, new0, new1);
    fetch(old0, old1, nk, nv);
    consume(c0, ok, ov);
    c0 = c1;
    c1 = c2;
    advance(c2);
    return c0.r >= n_out;
  };
  while (true) {
    if (round(ida0, ida1, idb0, idb1, ka, va, kb2, vb2)) break;
    if (round(idb0, idb1, ida0, ida1, kb2, vb2, ka, va)) break;
    if (round(ida0, ida1, idb0, idb1, ka, va, kb2, vb2)) break;
    if (round(idb0, idb1, ida0, ida1, kb2, vb2, ka, va)) break;
  }
}

// Rows without merging (no member lists exist): output row w is a copy of its conserved row.
template <typename T, int D>
__global__ void __launch_bounds__(256) copy_rows_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  constexpr int LPR = TL::kChunksPerRow;
  const long long piece = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long w = a.total_slots - 1 - piece / LPR;
  if (w < 0) return;
  const int cc = (int)(piece % LPR);
  const size_t src = (size_t)a.sel_idx[w] * TL::kRowBytes + cc * 16, dst = (size_t)w * TL::kRowBytes + cc * 16;
  store16_stream(a.k_out + dst, load16_stream(a.k + src));
  store16_stream(a.v_out + dst, load16_stream(a.v + src));
}

// ------------------------------------------------------------------------------------------ launch

static MergeArgs make_args(const Plan& p, const Buffers& b) {
  MergeArgs a;
  a.k = static_cast<const char*>(b.k);
  a.v = static_cast<const char*>(b.v);
  a.k_out = static_cast<char*>(b.k_out);
  a.v_out = static_cast<char*>(b.v_out);
  a.inv_norm = reinterpret_cast<const float*>(b.ws + p.off_inv_norm);
  a.alloc = reinterpret_cast<const int32_t*>(b.ws + p.off_alloc);
  a.off = reinterpret_cast<const int64_t*>(b.ws + p.off_layer_off);
  a.sel_idx = reinterpret_cast<const int32_t*>(b.ws + p.off_sel_idx);
  a.sel_inv_norm = reinterpret_cast<const float*>(b.ws + p.off_sel_inv);
  a.less_idx = reinterpret_cast<const int32_t*>(b.ws + p.off_less_idx);
  a.less_slot = reinterpret_cast<int32_t*>(b.ws + p.off_less_slot);
  a.sort_key[0] = reinterpret_cast<int32_t*>(b.ws + p.off_sort_a);
  a.sort_val[0] = reinterpret_cast<int32_t*>(b.ws + p.off_sort_b);
  a.sort_key[1] = reinterpret_cast<int32_t*>(b.ws + p.off_sort_c);
  a.sort_val[1] = reinterpret_cast<int32_t*>(b.ws + p.off_sort_d);
  a.seg_beg = reinterpret_cast<int32_t*>(b.ws + p.off_seg_beg);
  a.seg_end = reinterpret_cast<int32_t*>(b.ws + p.off_seg_end);
  a.merge_assign = b.merge_assign;
  a.L = p.L; a.Hkv = p.Hkv; a.T = p.T; a.flags = p.flags;
  a.total_slots = (long long)p.B * p.Hkv;
  a.use_resident = 0;
  a.merge_members = !((p.flags & MEDA_FLAG_NO_MERGE) || p.B == (int64_t)p.L * p.T);
  a.n_members = (int)(((int64_t)p.L * p.T - p.B) * p.Hkv);
  return a;
}

template <typename T, int D>
static hipError_t launch_sim_t(const Plan& p, MergeArgs a, hipStream_t s) {
  const unsigned nrb = (p.T + kSimRows - 1) / kSimRows, pairs = (unsigned)(p.L * p.Hkv);
  // one resident-set workgroup occupies a whole CU: only worth it with at least one per CU
  a.use_resident = (resident_capacity<T, D>() > 0 && pairs >= 256u) ? 1 : 0;
  dim3 grid(8u * nrb * ((pairs + 7u) / 8u));
  hipLaunchKernelGGL((similarity_argmax_kernel<T, D>), grid, dim3(kSimWaves * 64), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!a.use_resident) return hipSuccess;
  auto res = similarity_resident_kernel<T, D>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(res), hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(res, dim3(pairs * kResSplit), dim3(kResThreads), kResLdsBytes, s, a);
  return hipGetLastError();
}

hipError_t launch_similarity(const Plan& p, const Buffers& b, hipStream_t s) {
  const MergeArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_sim_t<bf16_t, 128>(p, a, s) : launch_sim_t<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_sim_t<float, 128>(p, a, s) : launch_sim_t<float, 64>(p, a, s);
}

hipError_t launch_segment_sort(const Plan& p, const Buffers& b, hipStream_t s) {
  const MergeArgs a = make_args(p, b);
  const int nthr = p.T >= 16384 ? 1024 : (p.T >= 4096 ? 512 : 256);  // measured at T = 4096: 512 threads 65 us, 1024 or 256 threads 75 us
  hipLaunchKernelGGL(segment_sort_kernel, dim3(p.Hkv, p.L), dim3(nthr), 0, s, a);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_merge_t(const Plan& p, const MergeArgs& a, hipStream_t s) {
  if (!a.merge_members) {
    const long long pieces = a.total_slots * Tile<T, D>::kChunksPerRow;
    hipLaunchKernelGGL((copy_rows_kernel<T, D>), dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
  }
  const long long waves = (a.total_slots + kMergeRowsPerWave - 1) / kMergeRowsPerWave;
  hipLaunchKernelGGL((merge_write_kernel<T, D>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_merge_write(const Plan& p, const Buffers& b, hipStream_t s) {
  const MergeArgs a = make_args(p, b);
  if (p.dtype == MEDA_BF16) return p.d == 128 ? launch_merge_t<bf16_t, 128>(p, a, s) : launch_merge_t<bf16_t, 64>(p, a, s);
  return p.d == 128 ? launch_merge_t<float, 128>(p, a, s) : launch_merge_t<float, 64>(p, a, s);
}

}  // namespace meda
