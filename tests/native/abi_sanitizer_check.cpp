// Host-side check of the C ABI's argument validation, meant to be built with -fsanitize=address,undefined on
// the host code (no GPU is touched: every call below returns before the first HIP call or only computes sizes).
// The kernel launchers are stubs: meda_api.hip is linked without the kernel translation units.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/meda.h"
#include "../../paper_2502_17599_amd/csrc/plan.hpp"

namespace meda {
#define MEDA_STUB(name) \
  hipError_t name(const Plan&, const Buffers&, hipStream_t) { fprintf(stderr, #name " must not be reached\n"); abort(); }
MEDA_STUB(launch_score_stats)
MEDA_STUB(launch_stats_combine)
MEDA_STUB(launch_score_accum)
MEDA_STUB(launch_allocate)
MEDA_STUB(launch_select)
MEDA_STUB(launch_similarity)
MEDA_STUB(launch_segment_sort)
MEDA_STUB(launch_merge_write)
}  // namespace meda

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static meda_params base_params() {
  meda_params p;
  memset(&p, 0, sizeof p);
  p.n_layers = 4; p.n_q_heads = 8; p.n_kv_heads = 2; p.head_dim = 128; p.seq_len = 1000; p.window = 32;
  p.total_budget = 4 * 250; p.recent_num = 3; p.recent_den = 4; p.dtype = MEDA_BF16; p.softmax_scale = 0.f;
  return p;
}

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }

int main() {
  meda_params p = base_params();
  const size_t need = meda_workspace_bytes(&p);
  EXPECT(need > 0 && need % 256 == 0);
  EXPECT(meda_workspace_bytes(nullptr) == 0);
  // regions lie inside the workspace
  for (int r = 0; r < 6; ++r) {
    size_t off = 0, bytes = 0;
    EXPECT(meda_workspace_region(&p, r, &off, &bytes) == MEDA_OK);
    EXPECT(off % 256 == 0 && off + bytes <= need);
  }
  size_t off = 0, bytes = 0;
  EXPECT(meda_workspace_region(&p, 99, &off, &bytes) == MEDA_ERR_INVALID_ARG);
  EXPECT(meda_workspace_region(&p, 0, nullptr, &bytes) == MEDA_ERR_INVALID_ARG);

  // random parameter sets, valid and invalid, extreme sizes included: no overflow, no crash; a positive size is
  // a multiple of 256 and grows with nothing negative inside
  for (int it = 0; it < 200000; ++it) {
    meda_params q = base_params();
    q.n_layers = (int32_t)(rnd() % 300) - 10;
    q.n_kv_heads = (int32_t)(rnd() % 40) - 2;
    q.n_q_heads = q.n_kv_heads > 0 ? q.n_kv_heads * (int32_t)(rnd() % 10) : (int32_t)(rnd() % 64) - 4;
    q.head_dim = (rnd() & 1) ? 128 : ((rnd() & 1) ? 64 : (int32_t)(rnd() % 300));
    q.seq_len = (rnd() & 7) ? (int32_t)(rnd() % 200000) : (int32_t)rnd();
    q.window = (int32_t)(rnd() % 200) - 5;
    q.total_budget = (rnd() & 3) ? (int64_t)q.n_layers * (int64_t)(rnd() % (q.seq_len > 0 ? q.seq_len : 1) + 1)
                                 : (int64_t)rnd() * (int64_t)rnd() - (1ll << 40);
    q.recent_num = (int32_t)(rnd() % 8) - 1; q.recent_den = (int32_t)(rnd() % 8) - 1;
    q.dtype = (int32_t)(rnd() % 4) - 1;
    q.flags = (int32_t)(rnd() % 8);
    q.n_seqs = (int32_t)(rnd() % 70) - 2;
    const size_t n = meda_workspace_bytes(&q);
    EXPECT(n % 256 == 0);
    if (n > 0) {
      for (int r = 0; r < 6; ++r) {
        EXPECT(meda_workspace_region(&q, r, &off, &bytes) == MEDA_OK);
        EXPECT(off + bytes <= n);
      }
    }
  }

  // meda_compress: everything below is rejected on the host
  alignas(256) static char buf[4096];
  void* ok = buf;
  int32_t* i32 = reinterpret_cast<int32_t*>(buf);
  int64_t* i64 = reinterpret_cast<int64_t*>(buf);
  const uint8_t* u8 = reinterpret_cast<const uint8_t*>(buf);
  EXPECT(meda_compress(nullptr, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need, nullptr) == MEDA_ERR_INVALID_ARG);
  EXPECT(meda_compress(&p, nullptr, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need, nullptr) == MEDA_ERR_INVALID_ARG);
  EXPECT(meda_compress(&p, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, nullptr, need, nullptr) == MEDA_ERR_WORKSPACE);
  EXPECT(meda_compress(&p, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, buf + 16, need, nullptr) == MEDA_ERR_WORKSPACE);
  EXPECT(meda_compress(&p, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need - 1, nullptr) == MEDA_ERR_WORKSPACE);
  EXPECT(meda_compress(&p, buf + 8, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need, nullptr) == MEDA_ERR_INVALID_ARG);
  meda_params bad = p; bad.total_budget = 4 * 31;
  EXPECT(meda_compress(&bad, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need, nullptr) == MEDA_ERR_BUDGET);
  bad = p; bad.head_dim = 96;
  EXPECT(meda_compress(&bad, ok, ok, ok, u8, ok, ok, i32, i64, nullptr, nullptr, nullptr, ok, need, nullptr) == MEDA_ERR_UNSUPPORTED);

  // strings for every code, names also outside the range
  for (int c = MEDA_OK; c <= MEDA_ERR_SCRATCH_LIMIT; ++c) EXPECT(meda_status_string((meda_status)c) != nullptr && strlen(meda_status_string((meda_status)c)) > 0);
  for (int ph = -2; ph < MEDA_N_PHASES + 2; ++ph) EXPECT(meda_phase_name(ph) != nullptr);
  EXPECT(meda_profile_enable(-1) == MEDA_ERR_INVALID_ARG && meda_profile_enable(2 + MEDA_N_PHASES) == MEDA_ERR_INVALID_ARG);
  double ms[MEDA_N_PHASES]; int32_t calls = -1;
  EXPECT(meda_profile_read(nullptr, &calls, 0) == MEDA_ERR_INVALID_ARG);
  EXPECT(meda_profile_read(ms, &calls, 1) == MEDA_OK && calls == 0);

  if (failures) { fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
  printf("abi sanitizer check ok\n");
  return 0;
}
