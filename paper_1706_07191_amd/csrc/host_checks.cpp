// Host-side checks of libbrsvd for a build whose host code is instrumented with the address and undefined-
// behaviour sanitizers (python -m paper_1706_07191_amd.build --host-asan).  Everything here runs without a
// GPU: argument validation, working-set sizing and block resolution, the launch planners of the two thin
// products over many shapes, and the failure paths of the calls that would touch a device -- on a machine
// without one they fail inside the runtime, and the library has to hand back a status and free what it took.
// The sanitizers turn an out-of-bounds access, a signed overflow or a leak on any of these paths into a
// non-zero exit status.
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "brsvd.h"
#include "brsvd_steps.h"

static int g_checks = 0, g_failed = 0;
#define CHECK(cond)                                                             \
  do {                                                                          \
    ++g_checks;                                                                 \
    if (!(cond)) { ++g_failed; std::printf("FAILED line %d: %s\n", __LINE__, #cond); } \
  } while (0)

static brsvd_params base_params() {
  brsvd_params p;
  std::memset(&p, 0, sizeof(p));
  p.m = 2000; p.n = 1000; p.k = 20; p.p = 10; p.q = 2; p.row_block = 512;
  return p;
}

// small deterministic generator (no library state)
static uint64_t g_state = 0x1706071910ull;
static uint64_t next_u64() {
  g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
  return g_state;
}
static int64_t uniform(int64_t lo, int64_t hi) { return lo + (int64_t)(next_u64() % (uint64_t)(hi - lo + 1)); }

int main() {
  uint64_t bytes = 0;
  brsvd_handle h = nullptr;

  // ---- argument validation ----
  CHECK(brsvd_workspace_bytes(nullptr, &bytes) == BRSVD_ERR_ARG);
  CHECK(brsvd_create(nullptr, &h) == BRSVD_ERR_ARG && h == nullptr);
  {
    brsvd_params p = base_params();
    CHECK(brsvd_workspace_bytes(&p, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_create(&p, nullptr) == BRSVD_ERR_ARG);
    struct { int field; int64_t value; } bad[] = {{0, 0}, {1, -1}, {2, 0}, {3, -1}, {4, -1}, {2, 600}, {0, 20}, {5, -5},
                                                  {6, 7}, {7, 5}, {8, 3}, {9, 9}, {10, 4}};
    for (auto& b : bad) {
      brsvd_params q = base_params();
      switch (b.field) {
        case 0: q.m = b.value; break;
        case 1: q.n = b.value; break;
        case 2: q.k = (int32_t)b.value; break;
        case 3: q.p = (int32_t)b.value; break;
        case 4: q.q = (int32_t)b.value; break;
        case 5: q.row_block = b.value; break;
        case 6: q.pass_mode = (int32_t)b.value; break;
        case 7: q.dtype = (int32_t)b.value; break;
        case 8: q.timing_level = (int32_t)b.value; break;
        case 9: q.a_location = (int32_t)b.value; break;
        case 10: q.orth_method = (int32_t)b.value; break;
      }
      CHECK(brsvd_workspace_bytes(&q, &bytes) == BRSVD_ERR_ARG);
      h = (brsvd_handle)0x1;
      CHECK(brsvd_create(&q, &h) == BRSVD_ERR_ARG && h == nullptr);
    }
    brsvd_params w = base_params();
    w.workspace = (void*)0x1004;          // misaligned
    w.workspace_bytes = 1ull << 30;
    CHECK(brsvd_create(&w, &h) == BRSVD_ERR_ARG && h == nullptr);
  }
  CHECK(brsvd_run(nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == BRSVD_ERR_ARG);
  CHECK(brsvd_run_f64(nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == BRSVD_ERR_ARG);
  CHECK(brsvd_run_alg2(nullptr, nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr, nullptr) == BRSVD_ERR_ARG);
  CHECK(brsvd_rpca_ialm(nullptr, nullptr, nullptr, 1, 0.1f, 1.f, 1.5f, 0.0, nullptr, nullptr, nullptr, nullptr, nullptr) ==
        BRSVD_ERR_ARG);
  CHECK(brsvd_norm2_power(nullptr, nullptr, 0, nullptr, 1, nullptr) == BRSVD_ERR_ARG);
  CHECK(brsvd_destroy(nullptr) == BRSVD_OK);
  CHECK(std::strcmp(brsvd_status_string(BRSVD_OK), "ok") == 0);
  for (int s = -6; s < 0; ++s) CHECK(std::strlen(brsvd_status_string(s)) > 2);
  CHECK(std::strcmp(brsvd_status_string(-99), "unknown status") == 0);

  // ---- working-set sizing and block resolution over many parameter sets ----
  for (int it = 0; it < 400; ++it) {
    brsvd_params p = base_params();
    p.m = uniform(1, 3) == 1 ? uniform(1, 400) : uniform(400, 300000);
    p.n = uniform(1, 3) == 1 ? uniform(1, 400) : uniform(400, 120000);
    const int64_t lmax = p.m < p.n ? p.m : p.n;
    const int64_t l = uniform(1, lmax < 512 ? lmax : 512);
    p.p = (int32_t)uniform(0, l - 1);
    p.k = (int32_t)(l - p.p);
    p.q = (int32_t)uniform(0, 3);
    p.dtype = (int32_t)uniform(0, 1);
    p.pass_mode = (int32_t)uniform(0, 1);
    p.a_location = (int32_t)uniform(0, 1);
    p.row_block = uniform(0, 3) == 0 ? 0 : uniform(1, p.m);
    if (p.a_location == BRSVD_A_HOST_PINNED && p.row_block == 0) p.device_budget_bytes = (uint64_t)uniform(1, 64) << 28;
    const int st = brsvd_workspace_bytes(&p, &bytes);
    CHECK(st == BRSVD_OK || st == BRSVD_ERR_BUDGET);
    if (st == BRSVD_OK) {
      const uint64_t esz = p.dtype == BRSVD_DTYPE_F64 ? 8 : 4;
      const uint64_t Lp = (uint64_t)(l + 15) / 16 * 16;
      CHECK(bytes >= 2 * (uint64_t)(p.m + p.n) * Lp * esz);              // the four thin panels
      if (p.device_budget_bytes) CHECK(bytes <= p.device_budget_bytes);
      brsvd_params tight = p;
      tight.device_budget_bytes = bytes - 1;
      if (p.row_block != 0) CHECK(brsvd_workspace_bytes(&tight, &bytes) == BRSVD_ERR_BUDGET);
    }
  }

  // ---- launch planners: every shape must give a plan with positive sizes and no overflow ----
  for (int it = 0; it < 3000; ++it) {
    const int64_t rows = uniform(1, 3) == 1 ? uniform(1, 300) : uniform(1, 2500000);
    const int64_t n = uniform(1, 3) == 1 ? uniform(1, 300) : uniform(1, 150000);
    const int32_t l = (int32_t)uniform(1, 512);
    const int32_t dtype = (int32_t)uniform(0, 1);
    int32_t out[12];
    CHECK(brsvd_gemm_plan(0, rows, n, l, 0, dtype, out) == BRSVD_OK);
    CHECK(out[0] > 0 && out[1] > 0 && out[2] > 0 && out[3] + out[4] == out[1] && out[9] > 0);
    const int64_t b = uniform(0, 1) ? 0 : uniform(1, rows);
    CHECK(brsvd_gemm_plan(1, rows, n, l, b, dtype, out) == BRSVD_OK);
    CHECK(out[2] > 0 && out[3] > 0 && out[4] > 0 && out[5] > 0 && out[6] == out[3] * out[4]);
    CHECK(brsvd_gemm_plan(2, rows, n, l, b, dtype, out) == BRSVD_OK);
    CHECK(out[0] >= 0 && out[1] >= 0 && out[2] >= 0 && out[3] >= 0);
  }
  {
    int32_t out[12];
    CHECK(brsvd_gemm_plan(0, 0, 10, 4, 0, 0, out) == BRSVD_ERR_ARG);
    CHECK(brsvd_gemm_plan(3, 10, 10, 4, 0, 0, out) == BRSVD_ERR_ARG);
    CHECK(brsvd_gemm_plan(0, 10, 10, 4, 0, 0, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_gemm_scratch_bytes(0, 10, 4) == 0 && brsvd_gemm_scratch_bytes(512, 1000, 30) > 0);
    CHECK(brsvd_orth_scratch_bytes(100, 600) == 0 && brsvd_small_svd_scratch_bytes(0) == 0);
    CHECK(brsvd_small_svd_scratch_bytes(512) >= 2ull * 512 * 512 * 8);
  }

  // ---- step calls: scratch that is missing, misaligned or too short is refused before any device call ----
  {
    void* one = (void*)0x100;
    CHECK(brsvd_gemm_an(nullptr, 0, 0, 0, nullptr, 0, nullptr, nullptr, 0, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_gemm_an((const float*)one, 64, 64, 64, (const float*)one, 8, (float*)one, one, 16, nullptr) == BRSVD_ERR_BUDGET);
    CHECK(brsvd_gemm_at((const float*)one, 64, 64, 64, (const float*)one, 8, (float*)one, 0, nullptr, 0, nullptr) ==
          BRSVD_ERR_BUDGET);
    CHECK(brsvd_orth(nullptr, 0, 0, 0, nullptr, nullptr, nullptr, 0, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_orth((float*)one, 100, 8, 0, nullptr, nullptr, one, 16, nullptr) == BRSVD_ERR_BUDGET);
    CHECK(brsvd_orth((float*)one, 100, 8, 0, nullptr, nullptr, (void*)0x108, 1 << 20, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_small_svd((const double*)one, 8, (double*)one, (double*)one, (double*)one, nullptr, nullptr, 1 << 20, nullptr) ==
          BRSVD_ERR_ARG);
    CHECK(brsvd_small_svd((const double*)one, 8, (double*)one, (double*)one, (double*)one, nullptr, one, 16, nullptr) ==
          BRSVD_ERR_BUDGET);
    CHECK(brsvd_small_svd_static((const double*)one, 513, (double*)one, (double*)one, (double*)one, nullptr, nullptr) ==
          BRSVD_ERR_BUDGET);
    CHECK(brsvd_small_svd_static(nullptr, 8, (double*)one, (double*)one, (double*)one, nullptr, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_philox_normal(1, 0, 0, 4, (float*)one, nullptr) == BRSVD_ERR_ARG);
    CHECK(brsvd_probe(0, nullptr, 16, nullptr, nullptr, nullptr) == BRSVD_ERR_ARG);
  }

  // ---- calls that reach the device: without one they must fail with a status and free everything ----
  {
    brsvd_params p = base_params();
    h = (brsvd_handle)0x1;
    const int st = brsvd_create(&p, &h);
    if (st == BRSVD_OK) {
      // a GPU is present: the handle is real; exercise destroy and stop here
      CHECK(h != nullptr && brsvd_destroy(h) == BRSVD_OK);
      std::printf("device present: failure paths of the runtime calls not exercised\n");
    } else {
      CHECK((st == BRSVD_ERR_ALLOC || st == BRSVD_ERR_HIP) && h == nullptr);
      brsvd_params hp = base_params();
      hp.a_location = BRSVD_A_HOST_PINNED;
      h = (brsvd_handle)0x1;
      const int st2 = brsvd_create(&hp, &h);
      CHECK((st2 == BRSVD_ERR_ALLOC || st2 == BRSVD_ERR_HIP) && h == nullptr);
      // caller-owned workspace: the failing create must not free it (it is not even a real allocation here)
      brsvd_params wp = base_params();
      CHECK(brsvd_workspace_bytes(&wp, &bytes) == BRSVD_OK);
      wp.workspace = (void*)0x10000;
      wp.workspace_bytes = bytes;
      h = (brsvd_handle)0x1;
      const int st3 = brsvd_create(&wp, &h);
      CHECK((st3 == BRSVD_ERR_ALLOC || st3 == BRSVD_ERR_HIP) && h == nullptr);
      wp.workspace_bytes = bytes - 1;
      CHECK(brsvd_create(&wp, &h) == BRSVD_ERR_BUDGET && h == nullptr);
      double sec = 0, work = 0;
      CHECK(brsvd_probe(0, (void*)0x10000, 1024, &sec, &work, nullptr) != BRSVD_OK);
    }
  }

  std::printf("host checks: %d run, %d failed\n", g_checks, g_failed);
  std::fflush(stdout);
  return g_failed ? 1 : 0;
}
