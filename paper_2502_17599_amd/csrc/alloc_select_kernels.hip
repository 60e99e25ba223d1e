// Layer budgets from the cross-modal entropies (Section 3.2 allocation equation, Appendix A.3,
// Section 4.3 for the recent : important split) and per-head token selection (Section 3.3: text
// prior, recent window, Top-N).
#include "device_utils.hpp"
#include "plan.hpp"

namespace meda {

// ------------------------------------------------------------------------------------ allocation
struct AllocArgs {
  const double* ent_part;  // [L][NT][2]: minus sum p log p over text rows / vision rows, per column tile
  const uint8_t* mask;
  int32_t* alloc;          // [L][4]: S, M, N, 0
  int64_t* off;            // [L+1]
  int32_t* layer_len;      // user outputs
  int64_t* layer_off;
  double* entropy;         // may be null
  int L, NT, T, W, R, num, den, flags;   // L layers and budget B of ONE sequence; W: recent window; R: scoring rows
  int N;                                 // sequences (one workgroup each)
  long long B;
};

__device__ __forceinline__ double clampd(double v, double lo, double hi) { return fmin(fmax(v, lo), hi); }

// One workgroup per sequence.  S_l = B * softmax_l(E_CM) when no bound is active; shares are kept inside
// [min(W,T), T] by water-filling (x_l = clamp(lambda * w_l), sum x_l = B) and rounded by largest
// remainder, so that sum_l S_l = B exactly.  All real arithmetic is double precision.
__global__ void __launch_bounds__(1024) allocate_kernel(AllocArgs a) {
  __shared__ double E[kMaxLayers], w[kMaxLayers], x[kMaxLayers], frac[kMaxLayers];
  __shared__ double kink[2 * kMaxLayers], filled[2 * kMaxLayers];
  __shared__ int S[kMaxLayers], order[kMaxLayers];
  __shared__ double s_lambda;
  const int tid = threadIdx.x, L = a.L;
  const double lo = (double)min(a.W, a.T), hi = (double)a.T, B = (double)a.B;
  // sequence n: its layers are the layers n*L .. n*L + L-1 of the batch, its output rows start at n*B
  const int n = blockIdx.x;
  a.ent_part += (size_t)n * L * a.NT * 2;
  a.mask += (size_t)n * a.T;
  if (a.entropy) a.entropy += (size_t)n * L;

  // scoring rows of each modality (the denominators of the two entropy means)
  int n_vis = 0;
  for (int r0 = 0; r0 < a.R; r0 += blockDim.x)
    n_vis += __syncthreads_count(r0 + tid < a.R && a.mask[a.T - a.R + r0 + tid] != 0);
  const int n_text = a.R - n_vis;
  // per-tile entropy partials of a layer are summed by one wave (lanes stride over the tiles)
  for (int l = tid >> 6; l < L; l += blockDim.x >> 6) {
    const double* p = a.ent_part + (size_t)l * a.NT * 2;
    double tv = 0.0, vt = 0.0;
    for (int t = tid & 63; t < a.NT; t += 64) {
      tv += p[2 * t];
      vt += p[2 * t + 1];
    }
    tv = wave_sum(tv);
    vt = wave_sum(vt);
    if ((tid & 63) == 0) {
      const double e = (n_text ? tv / n_text : 0.0) + (n_vis ? vt / n_vis : 0.0);
      E[l] = e;
      if (a.entropy) a.entropy[l] = e;
    }
  }
  __syncthreads();

  const bool uniform = (a.flags & MEDA_FLAG_UNIFORM_BUDGET) != 0;
  if (tid < L) {
    double emax = E[0];
    for (int i = 1; i < L; ++i) emax = fmax(emax, E[i]);
    w[tid] = uniform ? 1.0 : exp(E[tid] - emax);
  }
  __syncthreads();
  // the filled amount sum_l clamp(lambda w_l) is piecewise linear in lambda with kinks at lo/w and hi/w
  for (int i = tid; i < 2 * L; i += blockDim.x) {
    const double b = (i < L) ? lo / w[i] : hi / w[i - L];
    double f = 0.0;
    for (int j = 0; j < L; ++j) f += clampd(b * w[j], lo, hi);
    kink[i] = b;
    filled[i] = f;
  }
  __syncthreads();
  if (tid == 0) {
    double upper = -1.0, lower = 0.0;
    for (int i = 0; i < 2 * L; ++i) {
      if (filled[i] >= B) {
        if (upper < 0.0 || kink[i] < upper) upper = kink[i];
      } else if (kink[i] > lower) {
        lower = kink[i];
      }
    }
    const double mid = 0.5 * (lower + upper);
    double wsum = 0.0;
    int n_lo = 0, n_hi = 0;
    for (int j = 0; j < L; ++j) {
      const double v = mid * w[j];
      if (v <= lo) ++n_lo;
      else if (v >= hi) ++n_hi;
      else wsum += w[j];
    }
    s_lambda = (wsum > 0.0) ? (B - lo * n_lo - hi * n_hi) / wsum : upper;
  }
  __syncthreads();
  if (tid < L) {
    double xv = clampd(s_lambda * w[tid], lo, hi);
    if (a.B == (long long)L * a.T) xv = hi;
    if (a.B == (long long)L * min(a.W, a.T)) xv = lo;
    const double fl = floor(xv);
    x[tid] = xv;
    frac[tid] = xv - fl;
    S[tid] = (int)clampd(fl, lo, hi);
  }
  __syncthreads();
  if (tid < L) {
    int rank = 0;
    const double f = frac[tid];
    for (int j = 0; j < L; ++j) rank += (frac[j] > f || (frac[j] == f && j < tid)) ? 1 : 0;
    order[rank] = tid;  // decreasing fractional part, ties towards the lower layer
  }
  __syncthreads();
  if (tid == 0) {
    long long sum = 0;
    for (int j = 0; j < L; ++j) sum += S[j];
    long long rest = a.B - sum;
    for (int round = 0; round < 4 && rest > 0; ++round)
      for (int r = 0; r < L && rest > 0; ++r) {
        const int lyr = order[r];
        if (S[lyr] < a.T) { ++S[lyr]; --rest; }
      }
    for (int round = 0; round < 4 && rest < 0; ++round)  // only reachable through rounding fuzz
      for (int r = L - 1; r >= 0 && rest < 0; --r) {
        const int lyr = order[r];
        if (S[lyr] > min(a.W, a.T)) { --S[lyr]; ++rest; }
      }
  }
  __syncthreads();
  if (tid < L) {
    const int s = S[tid];
    const int m = max(min(a.W, s), (int)(((long long)s * a.num) / a.den));
    long long o = (long long)n * a.B;
    for (int j = 0; j < tid; ++j) o += S[j];
    const int lv = n * L + tid;  // layer of the batch
    a.alloc[4 * lv + 0] = s;
    a.alloc[4 * lv + 1] = m;
    a.alloc[4 * lv + 2] = s - m;
    // layers ranked by decreasing budget (ties: lower layer first), for kernels that launch the
    // longest workgroups first; in a batch the ranks of the sequences are interleaved (rank r of
    // sequence n is entry r*N + n), which keeps the order of one sequence and is decreasing on average
    int rank = 0;
    for (int j = 0; j < L; ++j) rank += (S[j] > s || (S[j] == s && j < tid)) ? 1 : 0;
    a.alloc[4 * (rank * a.N + n) + 3] = lv;
    a.off[lv] = o;
    a.layer_len[lv] = s;
    a.layer_off[(size_t)n * (L + 1) + tid] = o;
    if (tid == L - 1) {
      if (n == a.N - 1) a.off[(size_t)a.N * L] = o + s;
      a.layer_off[(size_t)n * (L + 1) + L] = o + s;
    }
  }
}

// ------------------------------------------------------------------------------------- selection
struct SelectArgs {
  const float* col_scores;  // [L][Hkv][T]
  const uint8_t* mask;
  const int32_t* alloc;
  const int64_t* off;
  int32_t* sel_idx;         // ragged [B*Hkv]: row ids (l*Hkv+g)*T + position
  float* sel_inv_norm;      // ragged [B*Hkv]: 1/|k| of every conserved key
  const float* inv_norm;    // [L][Hkv][T]
  int32_t* sel_idx_user;    // may be null
  int32_t* less_idx;        // ragged [(L*T-B)*Hkv]: row ids
  int32_t* merge_assign;    // may be null, [L][Hkv][T]
  int L, Hkv, T, no_merge;
  int Lseq;                 // layers per sequence (the mask is per sequence)
};

constexpr int kSelMaxThreads = 1024;
constexpr int kSelBatch = 4;  // loads a thread has in flight in the counting passes
constexpr int kSelMaxWaves = kSelMaxThreads / 64;

// Exclusive rank of a one-bit flag over the workgroup (ballots inside a wave, wave totals in LDS).
// `totals` has 2*kSelWaves ints; `slot` selects which half.  Returns rank; *block_total = number of set flags.
__device__ __forceinline__ int flag_rank_in_wave(bool flag, int lane, int* wave_total) {
  const unsigned long long b = __ballot(flag);
  *wave_total = __popcll(b);
  return __popcll(b & ((1ull << lane) - 1ull));
}

// grid (Hkv, L).  Adding max(A_s) to every text score puts all text candidates above all vision
// candidates and keeps the order inside each modality, so the Top-N of the boosted scores is:
// all text candidates plus the best vision ones if N exceeds the number of text candidates, else
// the best N text candidates.  The order inside one modality is found exactly on the unboosted
// fp32 scores (no bits are lost to the addition) with a 4 x 8-bit radix select on their bit
// patterns (scores are >= 0, so the unsigned order of the bits is the order of the values); equal
// scores go to the smaller position.
template <int kSelItems>  // consecutive positions a thread takes per iteration of the output pass
__global__ void __launch_bounds__(kSelMaxThreads) select_kernel(SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int wtot[2][kSelMaxWaves];
  __shared__ int s_red[kSelMaxWaves];
  __shared__ unsigned s_prefix;
  __shared__ int s_remaining;

  const int g = blockIdx.x, l = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kSelThreads = blockDim.x, kSelWaves = kSelThreads >> 6;
  const int T = a.T;
  const uint8_t* mask = a.mask + (size_t)(l / a.Lseq) * T;  // this layer's sequence
  const int S = a.alloc[4 * l + 0], M = a.alloc[4 * l + 1], N = a.alloc[4 * l + 2];
  const int ncand = T - M;
  const long long off_l = a.off[l];
  const int head_row0 = (l * a.Hkv + g) * T;  // row id of position 0 of this (layer, head)
  const float* scores = a.col_scores + (size_t)head_row0;
  const size_t c_base = (size_t)off_l * a.Hkv + (size_t)g * S;
  const size_t less_base = ((size_t)l * T - (size_t)off_l) * a.Hkv + (size_t)g * (T - S);

  // number of text candidates (kSelBatch loads in flight per thread: a pass over the scores of one head is bound by
  // the latency of its loads, not by their bytes)
  int cnt = 0;
  for (int j0 = tid; j0 < ncand; j0 += kSelBatch * kSelThreads) {
    uint8_t mk[kSelBatch];
#pragma unroll
    for (int i = 0; i < kSelBatch; ++i) mk[i] = mask[min(j0 + i * kSelThreads, ncand - 1)];
#pragma unroll
    for (int i = 0; i < kSelBatch; ++i) cnt += (j0 + i * kSelThreads < ncand && mk[i] == 0) ? 1 : 0;
  }
  cnt = wave_sum(cnt);
  if (lane == 0) s_red[wave] = cnt;
  __syncthreads();
  int n_text = 0;
  for (int i = 0; i < kSelWaves; ++i) n_text += s_red[i];

  const bool pick_text = N <= n_text;            // class in which the cut falls
  const int K = pick_text ? N : N - n_text;      // how many of that class are taken
  const bool other_taken = !pick_text;           // vision cut: every text candidate is taken
  const uint8_t cls = pick_text ? 0 : 1;

  unsigned threshold = 0xffffffffu;
  int ties_taken = 0;
  if (K > 0) {
    if (tid == 0) { s_prefix = 0u; s_remaining = K; }
    unsigned prefix_mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      const unsigned prefix = s_prefix;
      for (int j0 = tid; j0 < ncand; j0 += kSelBatch * kSelThreads) {
        uint8_t mk[kSelBatch];
        unsigned key[kSelBatch];
#pragma unroll
        for (int i = 0; i < kSelBatch; ++i) {
          const int j = min(j0 + i * kSelThreads, ncand - 1);
          mk[i] = mask[j];
          key[i] = __float_as_uint(scores[j]);
        }
#pragma unroll
        for (int i = 0; i < kSelBatch; ++i) {
          if (j0 + i * kSelThreads < ncand && (mk[i] != 0) == (cls != 0) && (key[i] & prefix_mask) == prefix)
            atomicAdd(&hist[(key[i] >> shift) & 255u], 1);
        }
      }
      __syncthreads();
      if (wave == 0) {
        // bins from the top: lane i looks at bins 255-4i .. 252-4i; the lane whose running count
        // first reaches `remaining` holds the digit of the K-th largest key
        const int remaining = s_remaining;
        const int b0 = 255 - 4 * lane;
        const int c0 = hist[b0], c1 = hist[b0 - 1], c2 = hist[b0 - 2], c3 = hist[b0 - 3];
        const int tot = c0 + c1 + c2 + c3;
        int inc = tot;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_up(inc, o, kWave);
          if (lane >= o) inc += t;
        }
        const int exc = inc - tot;
        if (exc < remaining && inc >= remaining) {
          int cum = exc, digit = b0;
          if (cum + c0 < remaining) {
            cum += c0; digit = b0 - 1;
            if (cum + c1 < remaining) {
              cum += c1; digit = b0 - 2;
              if (cum + c2 < remaining) { cum += c2; digit = b0 - 3; }
            }
          }
          s_remaining = remaining - cum;
          s_prefix = prefix | ((unsigned)digit << shift);
        }
      }
      prefix_mask |= 255u << shift;
      __syncthreads();
    }
    threshold = s_prefix;
    ties_taken = s_remaining;
  }

  // ordered output: conserved positions ascending, the rest ascending.  A thread takes kSelItems consecutive
  // positions per iteration (two barriers per kSelItems * blockDim positions); their mask, score and 1/|k| are
  // requested one iteration ahead, so that the barriers do not sit behind the loads.
  int run_c = 0, run_tie = 0;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  uint8_t mk_n[kSelItems];
  unsigned key_n[kSelItems];
  float inv_n[kSelItems];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
      const int jj = min(j0 + i, T - 1);
      mk_n[i] = mask[jj];
      key_n[i] = __float_as_uint(scores[jj]);
      inv_n[i] = a.inv_norm[head_row0 + jj];
    }
  };
  fetch(tid * kSelItems);
  for (int base = 0; base < T; base += kSelItems * kSelThreads) {
    const int j0 = base + tid * kSelItems;
    uint8_t mk[kSelItems];
    unsigned key[kSelItems];
    float inv[kSelItems];
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
      mk[i] = mk_n[i];
      key[i] = key_n[i];
      inv[i] = inv_n[i];
    }
    fetch(j0 + kSelItems * kSelThreads);
    bool valid[kSelItems], in_cls[kSelItems], is_tie[kSelItems], above[kSelItems];
    int tie_before = 0, tie_wave = 0;
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
      const int j = j0 + i;
      valid[i] = j < T;
      in_cls[i] = is_tie[i] = above[i] = false;
      if (valid[i] && j < ncand) {
        in_cls[i] = (mk[i] != 0) == (cls != 0);
        if (in_cls[i]) {
          above[i] = key[i] > threshold;
          is_tie[i] = key[i] == threshold;
        }
      }
      const unsigned long long b = __ballot(is_tie[i]);
      tie_before += __popcll(b & lt_mask);  // ties at the positions of the lanes below
      tie_wave += __popcll(b);
    }
    if (lane == 0) wtot[0][wave] = tie_wave;
    __syncthreads();
    int tie_rank = run_tie + tie_before, tie_total = 0;
    for (int i = 0; i < kSelWaves; ++i) {
      const int v = wtot[0][i];
      tie_rank += (i < wave) ? v : 0;
      tie_total += v;
    }
    bool sel[kSelItems];
    int sel_before = 0, sel_wave = 0;
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
      const int j = j0 + i;
      sel[i] = valid[i] && (j >= ncand || (in_cls[i] ? (above[i] || (is_tie[i] && tie_rank < ties_taken)) : other_taken));
      tie_rank += is_tie[i] ? 1 : 0;  // this thread's positions are consecutive
      const unsigned long long b = __ballot(sel[i]);
      sel_before += __popcll(b & lt_mask);
      sel_wave += __popcll(b);
    }
    if (lane == 0) wtot[1][wave] = sel_wave;
    __syncthreads();
    int pos_c = run_c + sel_before, sel_total = 0;
    for (int i = 0; i < kSelWaves; ++i) {
      const int v = wtot[1][i];
      pos_c += (i < wave) ? v : 0;
      sel_total += v;
    }
#pragma unroll
    for (int i = 0; i < kSelItems; ++i) {
      const int j = j0 + i;  // pos_c conserved positions lie before j
      if (sel[i]) {
        a.sel_idx[c_base + pos_c] = head_row0 + j;
        a.sel_inv_norm[c_base + pos_c] = inv[i];
        if (a.sel_idx_user) a.sel_idx_user[c_base + pos_c] = j;
        if (a.merge_assign) a.merge_assign[head_row0 + j] = pos_c;
        ++pos_c;
      } else if (valid[i]) {
        a.less_idx[less_base + (j - pos_c)] = head_row0 + j;
        if (a.merge_assign && a.no_merge) a.merge_assign[head_row0 + j] = -1;
      }
    }
    run_c += sel_total;
    run_tie += tie_total;
  }
}

// ------------------------------------------------------------------------------------------ launch

hipError_t launch_allocate(const Plan& p, const Buffers& b, hipStream_t s) {
  AllocArgs a;
  a.ent_part = reinterpret_cast<const double*>(b.ws + p.off_ent_part);
  a.mask = b.mask;
  a.alloc = reinterpret_cast<int32_t*>(b.ws + p.off_alloc);
  a.off = reinterpret_cast<int64_t*>(b.ws + p.off_layer_off);
  a.layer_len = b.layer_len;
  a.layer_off = b.layer_off;
  a.entropy = b.entropy;
  a.L = p.Lseq; a.NT = p.NTk; a.T = p.T; a.W = p.W; a.R = p.R; a.num = p.num; a.den = p.den; a.flags = p.flags;
  a.N = p.N;
  a.B = p.B / p.N;
  hipLaunchKernelGGL(allocate_kernel, dim3(p.N), dim3(1024), 0, s, a);  // 16 waves share the per-layer sums of the entropy partials
  return hipGetLastError();
}

hipError_t launch_select(const Plan& p, const Buffers& b, hipStream_t s) {
  SelectArgs a;
  a.col_scores = reinterpret_cast<const float*>(b.ws + p.off_col_scores);
  a.mask = b.mask;
  a.alloc = reinterpret_cast<const int32_t*>(b.ws + p.off_alloc);
  a.off = reinterpret_cast<const int64_t*>(b.ws + p.off_layer_off);
  a.sel_idx = reinterpret_cast<int32_t*>(b.ws + p.off_sel_idx);
  a.sel_inv_norm = reinterpret_cast<float*>(b.ws + p.off_sel_inv);
  a.inv_norm = reinterpret_cast<const float*>(b.ws + p.off_inv_norm);
  a.sel_idx_user = b.sel_idx_user;
  a.less_idx = reinterpret_cast<int32_t*>(b.ws + p.off_less_idx);
  a.merge_assign = b.merge_assign;
  a.L = p.L; a.Hkv = p.Hkv; a.T = p.T; a.no_merge = (p.flags & MEDA_FLAG_NO_MERGE) ? 1 : 0;
  a.Lseq = p.Lseq;
  const int nthr = p.T >= 16384 ? 1024 : (p.T >= 4096 ? 512 : 256);
  // long sequences: four positions per thread and iteration in the output pass (a quarter of the barriers); short
  // ones have too few iterations for that to pay
  if (p.T >= 16384) hipLaunchKernelGGL(select_kernel<4>, dim3(p.Hkv, p.L), dim3(nthr), 0, s, a);
  else hipLaunchKernelGGL(select_kernel<1>, dim3(p.Hkv, p.L), dim3(nthr), 0, s, a);
  return hipGetLastError();
}

}  // namespace meda
