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
  char* packed_k;           // ragged [B*Hkv][d]: the conserved keys, copied once so that tiles of them are contiguous
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
constexpr int kResSplit = 1;  // 2 and 3 parts per pair (more, shorter workgroups) measured slower; so did giving this
                             // kernel only as many layers as fill whole rounds of one workgroup per CU

// conserved keys (a multiple of 32) that fit: one padded row and one 1/|k| each
template <typename T, int D>
constexpr int resident_capacity() {
  // rows above 256 bytes would need more registers per wave than eight waves per CU leave
  return Tile<T, D>::kRowBytes > 256 ? 0 : kResLdsBytes / (Tile<T, D>::kStride + 4) / 32 * 32;
}

// u_ij = (k_i . k_j)/(|k_i| |k_j|): the raw keys are multiplied (bf16 products are exact in the fp32
// accumulator), the factor 1/|k_j| of the conserved key is applied to the accumulator, and the positive
// factor 1/|k_i| of the row is dropped because it cannot change the argmax over j.  Ties go to the lower slot.
//
// A wave keeps 64 less-important rows as two B-operand fragments in registers and takes the conserved keys of
// its (layer, head) from LDS as A operands, 32 slots (one block) at a time.  With the conserved keys as
// operand A, a lane owns ONE row and sees 16 candidate slots per block in its 16 accumulator registers: the
// running best of the row is one value per lane and the block maximum is a max3 tree.
//
// Running best of one row (one lane) over the blocks it has seen: the best value, the first slot of
// the block that produced it and that block's 16 scaled products.  Keeping the products postpones the
// search for the winning register to the end of the kernel: per block only the maximum is formed
// (max3 tree), and the 16 products are copied in blocks where some lane of the wave improved.
struct RowBest {
  float best;
  int slot0;
  float u[16];
};

__device__ __forceinline__ void row_best_init(RowBest& rb) {
  rb.best = -INFINITY;
  rb.slot0 = 0;
#pragma unroll
  for (int r = 0; r < 16; ++r) rb.u[r] = -INFINITY;
}

// The 1/|k_j| of this lane's 16 slots of a block (iv_lds points at the block's entries of this lane group: slot
// r4*8 + i of the group sits at iv_lds[r4*8 + i]).
__device__ __forceinline__ void load_inv(float (&iv)[16], const float* iv_lds) {
#pragma unroll
  for (int r4 = 0; r4 < 4; ++r4) {
    const float4 v = *reinterpret_cast<const float4*>(iv_lds + r4 * 8);
    iv[r4 * 4 + 0] = v.x;
    iv[r4 * 4 + 1] = v.y;
    iv[r4 * 4 + 2] = v.z;
    iv[r4 * 4 + 3] = v.w;
  }
}

// Scales the 16 products of this lane by the 1/|k_j| of their slots and returns their maximum.
__device__ __forceinline__ float scale_max(f32x16_t& p, const float (&iv)[16]) {
#pragma unroll
  for (int r = 0; r < 16; ++r) p[r] *= iv[r];
  float bm = fmaxf(fmaxf(p[0], p[1]), p[2]);
#pragma unroll
  for (int r = 3; r < 15; r += 2) bm = fmaxf(fmaxf(bm, p[r]), p[r + 1]);
  return fmaxf(bm, p[15]);
}

__device__ __forceinline__ void keep_if_improved(const f32x16_t& u, float bm, int slot0, RowBest& rb) {
  const bool improved = bm > rb.best;  // strict: an equal value in a later block does not replace
  if (__ballot(improved) != 0ull) {
#pragma unroll
    for (int r = 0; r < 16; ++r) rb.u[r] = improved ? u[r] : rb.u[r];
    rb.best = improved ? bm : rb.best;
    rb.slot0 = improved ? slot0 : rb.slot0;
  }
}

// Slot of the row's best: the lowest register of the saved block that holds the maximum.  `best` is the maximum of
// exactly these 16 values (the max3 tree of keep_if_improved's caller), so one of them compares equal to it; walking
// down from register 15 leaves the lowest such register.  (Not a search for the smallest best - u[r] through a packed
// integer key: a key of 32 bits has no room for all 31 bits of a non-negative float beside the 4 bits of r, and
// whichever float bits are dropped, some nonzero difference then packs to the same key as the zero of the maximum.)
__device__ __forceinline__ int row_best_slot(const RowBest& rb, int kg) {
  int ridx = 15;
#pragma unroll
  for (int r = 14; r >= 0; --r) ridx = (rb.u[r] == rb.best) ? r : ridx;
  return rb.slot0 + (ridx >> 2) * 8 + kg * 4 + (ridx & 3);
}

// The two lane groups of a wave saw disjoint slots of the same row: the better one, ties -> lower slot.
__device__ __forceinline__ int row_best_merge(const RowBest& rb, int kg) {
  const int mine = row_best_slot(rb, kg);
  const float ov = __shfl_xor(rb.best, 32, kWave);
  const int oi = __shfl_xor(mine, 32, kWave);
  const bool take = ov > rb.best || (ov == rb.best && oi < mine);
  return take ? oi : mine;
}

// One block of 32 conserved slots against the wave's two row fragments: fragment and 1/|k_j| from LDS, both
// products (the two accumulator chains alternate), then scaling, maxima and the copy of an improved block.
// With two waves per SIMD one wave's vector phase runs beside the other's matrix phase.  (Variants that
// interleave the vector work of the previous block with the matrix instructions inside one wave, by hand or
// through the scheduler, measured the same or slower on every workload: under random operands the chip is
// limited by power, its clock drops to about 1.5 GHz in this kernel, and what counts is the number of
// instructions and LDS bytes per block, not their order.)
// The last tile of a (layer, head) is padded with copies of the last conserved key: a copy ties with the
// original and the tie rules (strict improvement, lowest register, lower slot between the lane groups)
// always prefer the original, so no slot needs masking and there is a single code path.
template <typename T, int D>
__device__ __forceinline__ void sim_block_products(const char* block, const unsigned (&coff)[Tile<T, D>::kFragChunks],
                                                   const Frag<T, D> (&lf)[2], f32x16_t (&acc)[2]) {
  Frag<T, D> cf;
#pragma unroll
  for (int c = 0; c < Tile<T, D>::kFragChunks; ++c) cf.c[c] = *reinterpret_cast<const uint4*>(block + coff[c]);
  acc[0] = acc_zero();
  acc[1] = acc_zero();
  mma<T, D>(acc[0], cf, lf[0]);
  mma<T, D>(acc[1], cf, lf[1]);
}

template <typename T, int D>
__device__ __forceinline__ void sim_block_simple(const char* block, const unsigned (&coff)[Tile<T, D>::kFragChunks],
                                                 const Frag<T, D> (&lf)[2], const float* iv_lds, int slot0, RowBest (&rb)[2]) {
  float iv[16];
  load_inv(iv, iv_lds);
  f32x16_t acc[2];
  sim_block_products<T, D>(block, coff, lf, acc);
  const float bm0 = scale_max(acc[0], iv), bm1 = scale_max(acc[1], iv);
  keep_if_improved(acc[0], bm0, slot0, rb[0]);
  keep_if_improved(acc[1], bm1, slot0, rb[1]);
}

// Tiled kernel: grid over (row block of 256, kv head, layer); 4 waves x 64 less-important rows.  The conserved
// keys stream through a ring of four LDS tiles of 64 slots, filled by asynchronous copies that go from global
// memory straight into LDS (no registers, no LDS store instructions): while tile t is multiplied, tile t+1 has
// landed, tile t+2 is landing and the copies of tile t+3 have just been issued, which gives every copy two tile
// times to arrive; one wait and one barrier per tile.
//
// LDS layout of a tile: 64 rows, unpadded, 16-byte chunk c of row r at position c ^ swz(r) of the row.  A copy
// instruction writes lane i's 16 bytes at (instruction base) + 16 i, so the rows cannot be padded; which global
// chunk a lane fetches is free, and the xor spreads the 16 rows a fragment load touches in one pass over all
// banks (rows of 256 bytes start at the same bank: swz(r) = r mod 16; two rows of 128 bytes share a bank
// line: swz(r) = (r / 2) mod 8).
// The 1/|k_j| of a tile are copied the same way (4 bytes per lane); every wave keeps its own copy, so all waves
// issue the same number of copies per tile and wait for the same count.
constexpr int kSimRing = 4;
constexpr int kSimInvRing = 8;

template <typename T, int D>
constexpr int sim_tiled_lds_bytes() {
  return kSimRing * kSimSlotTile * Tile<T, D>::kRowBytes + kSimInvRing * kSimWaves * kSimSlotTile * (int)sizeof(float);
}

template <typename T, int D>
__global__ void __launch_bounds__(kSimWaves * 64, (Tile<T, D>::kRowBytes <= 256 ? 2 : 1)) similarity_argmax_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  constexpr int CPR = TL::kChunksPerRow;
  constexpr int NC = TL::kFragChunks;
  constexpr int RPI = 64 / CPR;                        // rows one copy instruction fills
  constexpr int PF = kSimSlotTile / RPI / kSimWaves;   // key copy instructions per wave and tile
  constexpr int NB = kSimSlotTile / 32;                // blocks per tile
  constexpr int KPT = PF + 1;                          // copies per wave and tile (keys and 1/|k|)
  constexpr int kTileBytes = kSimSlotTile * TL::kRowBytes;
  static_assert(kSimSlotTile % (RPI * kSimWaves) == 0, "the copy instructions must tile the rows of a tile evenly");
  extern __shared__ __align__(16) char smem[];
  char* ctile = smem;                                                       // [kSimRing][64 rows]
  float* cinv = reinterpret_cast<float*>(smem + kSimRing * kTileBytes);     // [kSimInvRing][waves][64]

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

  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, kg = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long off_l = a.off[l];
  const size_t cbase = (size_t)off_l * a.Hkv + (size_t)g * S;
  // the bases of the asynchronous copies below must sit in scalar registers: said explicitly, not left to what the
  // compiler can prove about the address arithmetic
  const float* sinv = uniform_ptr(a.sel_inv_norm + cbase);
  const char* pk = uniform_ptr(a.packed_k + cbase * TL::kRowBytes);  // this pair's conserved keys, contiguous
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
  row_best_init(rb[0]);
  row_best_init(rb[1]);
  Frag<T, D> lf[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) frag_load(lf[s], kbase + (size_t)lrow[s] * TL::kRowBytes, kg);

  // Copy instruction j of this wave fills the rows (wave * PF + j) * RPI .. + RPI-1 of a tile: this lane brings
  // one 16-byte chunk of row crow_r + j * RPI.  Slots past the end of the set repeat the last conserved key (see
  // sim_block_simple).  Tiles past the last one repeat it too (they are never read; issuing them keeps the number
  // of copies in flight the same in every iteration).
  const int ntiles = (S + kSimSlotTile - 1) / kSimSlotTile;
  const int crow_r = wave * PF * RPI + lane / CPR;
  const unsigned lds_ring = (unsigned)(size_t)ctile, lds_inv = (unsigned)(size_t)cinv;
  auto issue_tile = [&](int t, int ring_slot) {  // tile t of the stream into slot ring_slot of the rings
    const int tc = min(t, ntiles - 1);
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int r = crow_r + j * RPI;   // row of the tile; its swizzle does not depend on the tile
      const int slot = min(tc * kSimSlotTile + r, S - 1);
      const unsigned goff = (unsigned)(slot * TL::kRowBytes + (((lane % CPR) ^ swizzle_of_row<T, D>(r)) * 16));
      async_copy16_to_lds(pk, goff, lds_ring + (unsigned)((ring_slot % kSimRing) * kTileBytes + (wave * PF + j) * 1024));
    }
    const unsigned goff4 = (unsigned)(min(tc * kSimSlotTile + lane, S - 1) * 4);
    const unsigned loff4 = (unsigned)((((ring_slot % kSimInvRing) * kSimWaves + wave) * kSimSlotTile) * 4);
    async_copy4_to_lds(sinv, goff4, lds_inv + loff4);
  };
  issue_tile(0, 0);
  issue_tile(1, 1);
  issue_tile(2, 2);

  // chunk c of this lane's fragment (chunk kg * NC + c of row n of a block) sits at (n * row bytes) +
  // 16 * ((kg * NC + c) ^ swz(n)) inside a block of 32 rows
  unsigned coff[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) coff[c] = (unsigned)(n * TL::kRowBytes + (((kg * NC + c) ^ swizzle_of_row<T, D>(n)) * 16));
  // block cb of the tile in ring slot rs: its rows and where its 1/|k_j| start in this wave's copy
  auto block_rows = [&](int rs, int cb) { return ctile + (rs % kSimRing) * kTileBytes + cb * 32 * TL::kRowBytes; };
  auto inv_index = [&](int rs, int cb) { return ((rs % kSimInvRing) * kSimWaves + wave) * kSimSlotTile + cb * 32; };

  async_copy_wait<KPT>();  // tiles 0 and 1 have landed (this wave's part)
  __syncthreads();         // every wave's part has
  issue_tile(3, 3);
  for (int t = 0; t < ntiles; ++t) {
    if (t > 0) {
      async_copy_wait<KPT>();    // this wave's part of tile t+1 has landed; tile t+2 may still be in flight
      __syncthreads();           // every wave's part has; and nobody reads tile t-1 any more
      issue_tile(t + 3, t + 3);  // into the buffer of tile t-1
    }
#pragma unroll
    for (int cb = 0; cb < NB; ++cb)
      sim_block_simple<T, D>(block_rows(t, cb), coff, lf, cinv + inv_index(t, cb) + kg * 4, (t * NB + cb) * 32, rb);
  }
  async_copy_wait<0>();  // nothing of this wave is still on its way into LDS when it ends

#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int bi = row_best_merge(rb[s], kg);
    const int ri = r0 + s * 32 + n;
    if (kg == 0 && ri < n_less) {
      a.less_slot[lbase + ri] = bi;
      if (a.merge_assign) a.merge_assign[less[ri]] = bi;
    }
  }
}

// Variant for layers whose conserved set fits into LDS: one workgroup keeps ALL conserved keys of its
// (layer, head) resident and every wave streams chunks of 64 less-important rows through registers.
// After the prologue there is no barrier: the waves run independently and the keys are read from HBM once.
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
  const float* sinv = a.sel_inv_norm + cbase;
  const char* pk = a.packed_k + cbase * TL::kRowBytes;  // this pair's conserved keys, contiguous
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
  // k-step i of a fragment takes the bytes [32 i + 16 kg, + 16) of its row: the two lane groups read adjacent
  // pieces, so a load instruction touches 32 cache lines instead of the 64 of the half-row mapping (this kernel
  // loads 64 rows per wave and chunk, all the time).  The conserved keys are read from LDS with the same mapping,
  // and any fixed order of the k-steps gives the same products.
  auto row_frag = [&](Frag<T, D>& f, const char* row_ptr) {
#pragma unroll
    for (int i = 0; i < TL::kFragChunks; ++i) f.c[i] = *reinterpret_cast<const uint4*>(row_ptr + i * 32 + kg * 16);
  };
  Frag<T, D> lf[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) row_frag(lf[s], kbase + (size_t)lrow[s] * TL::kRowBytes);

  // Prologue: the conserved keys into LDS.  The set is padded to a multiple of 32 slots with
  // copies of the last key (a copy can never win a tie against the original, see sim_block_simple).
  const int S_pad = (S + 31) & ~31;
  char* ckeys = smem;
  float* cinv = reinterpret_cast<float*>(smem + (size_t)S_pad * TL::kStride);
  // All pieces of the set are requested before the first one is stored (one memory latency for the whole set; at
  // most kMaxPieces 16-byte pieces per thread; the bounds are the same for every thread of the workgroup, so the
  // tests are scalar branches).  The batch is an array of a native vector type: as an array of uint4 the compiler
  // kept it in scratch memory.
  constexpr int kMaxPieces = (resident_capacity<T, D>() * CPR + kResThreads - 1) / kResThreads;
  const int n_pieces = S_pad * CPR;
  {
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    u32x4_t v[kMaxPieces > 0 ? kMaxPieces : 1];
#pragma unroll
    for (int i = 0; i < kMaxPieces; ++i) {
      if (i * kResThreads < n_pieces) {
        const int p = min(tid + i * kResThreads, n_pieces - 1);
        v[i] = *reinterpret_cast<const u32x4_t*>(pk + (unsigned)(min(p / CPR, S - 1) * TL::kRowBytes + (p % CPR) * 16));
      }
    }
#pragma unroll
    for (int i = 0; i < kMaxPieces; ++i) {
      if (i * kResThreads < n_pieces) {
        const int p = min(tid + i * kResThreads, n_pieces - 1);  // a repeated piece: the same bytes to the same place
        *reinterpret_cast<u32x4_t*>(ckeys + (p / CPR) * TL::kStride + (p % CPR) * 16) = v[i];
      }
    }
  }
  for (int sl = tid; sl < S_pad; sl += kResThreads) cinv[sl] = sinv[min(sl, S - 1)];
  __syncthreads();

  const int nblocks = S_pad / 32;
  unsigned coff[TL::kFragChunks];   // chunk c of this lane's fragment inside a block of 32 padded rows
#pragma unroll
  for (int c = 0; c < TL::kFragChunks; ++c) coff[c] = (unsigned)(n * TL::kStride + c * 32 + kg * 16);
  auto block_base = [&](int b) { return ckeys + b * 32 * TL::kStride; };
  auto block_inv = [&](int b) { return cinv + b * 32 + kg * 4; };
  while (c < n_chunks) {
    // the rows of the wave's next chunk and the row ids of the one after it are in flight while
    // this chunk is multiplied (past the last chunk they repeat the last row and are dropped)
    const int r0 = c * kSimRowsPerWave;
    Frag<T, D> lfn[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) row_frag(lfn[s], kbase + (size_t)nrow[s] * TL::kRowBytes);
    int nnrow[2];
    chunk_rows(c + 2 * kChunkStep, nnrow);
    RowBest rb[2];
    row_best_init(rb[0]);
    row_best_init(rb[1]);
    for (int b = 0; b < nblocks; ++b) sim_block_simple<T, D>(block_base(b), coff, lf, block_inv(b), b * 32, rb);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int bi = row_best_merge(rb[s], kg);
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

// ------------------------------------------------------------------------ conserved keys, packed
// Output row w of the ragged cache is the conserved key sel_idx[w]; the rows of one (layer, head) are
// consecutive in w.  Copying them once into that order makes every tile of conserved keys the similarity
// kernels stream a contiguous block (which a lane-addressed asynchronous copy into LDS needs).
// 256 rows per workgroup.
constexpr int kPackRows = 256;
template <typename T, int D>
__global__ void __launch_bounds__(256) pack_conserved_kernel(MergeArgs a) {
  using TL = Tile<T, D>;
  constexpr int LPR = TL::kChunksPerRow;   // lanes per row
  constexpr int RPP = 256 / LPR;           // rows per pass
  constexpr int U = 4;                     // passes whose loads are in flight together
  static_assert(kPackRows % (RPP * U) == 0, "passes must tile the workgroup's rows");
  const int tid = threadIdx.x;
  const long long w0 = (long long)blockIdx.x * kPackRows, total = a.total_slots;
  const int sub = tid / LPR, cc = tid - sub * LPR;
  for (int r0 = 0; r0 < kPackRows; r0 += RPP * U) {
    int idx[U];
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) idx[u] = a.sel_idx[min(w0 + r0 + u * RPP + sub, total - 1)];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load16_stream(a.k + (size_t)idx[u] * TL::kRowBytes + cc * 16);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long w = w0 + r0 + u * RPP + sub;
      if (w < total) *reinterpret_cast<uint4*>(a.packed_k + (size_t)w * TL::kRowBytes + cc * 16) = v[u];
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
constexpr int kSortBits = 5;  // 6-bit digits (one pass fewer on long sets) measured slower: wave 0's prefix over the waves per tile weighs more
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
          if (wave == 0) {  // (a scan spread over all waves, 16 lanes per digit, measured slower than this walk by one wave)
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
  a.packed_k = b.ws + p.off_packed_k;
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
  hipLaunchKernelGGL((pack_conserved_kernel<T, D>), dim3((unsigned)((a.total_slots + kPackRows - 1) / kPackRows)),
                     dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid(8u * nrb * ((pairs + 7u) / 8u));
  constexpr int kTiledLds = sim_tiled_lds_bytes<T, D>();
  auto tiled = similarity_argmax_kernel<T, D>;
  if (kTiledLds > 64 * 1024) {
    e = allow_dynamic_lds(tiled, kTiledLds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(tiled, grid, dim3(kSimWaves * 64), kTiledLds, s, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!a.use_resident) return hipSuccess;
  auto res = similarity_resident_kernel<T, D>;
  e = allow_dynamic_lds(res, kResLdsBytes);
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
