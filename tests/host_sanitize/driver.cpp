// Sanitizer driver for the host layer of libamskv (csrc/amskv_api.cpp): built by tests/test_host_sanitize.py
// with -fsanitize=address,undefined together with amskv_api.cpp, it walks plan-only caches (no device memory)
// through every host-side call of the C ABI -- the scale-window policies and schedules of the host layout
// tests, the token-budget mode (Algorithms 1 and 2 with both outcomes of the Eq. 3 test forced by the
// threshold), the error paths -- and checks structural invariants on the way.  Parity with the oracle is the
// business of tests/test_host_layout.py; this program exists so that an out-of-bounds access, a use after
// free or undefined behaviour in the metadata code stops a test run.
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <vector>

#include "amskv_internal.hpp"

// ---- the device side is not part of this build: the launchers and the two runtime calls the host layer
// uses are stubs that fail loudly if the plan-only paths ever reach them
namespace amskv {
hipError_t launch_attend_bf16(const void*, void*, void*, void*, int, int, int, int64_t, const SegTable&, const ExtKV&,
                              const CallerIo&, float, hipStream_t) { std::abort(); }
hipError_t launch_attend_f32(const void*, void*, void*, void*, int, int, int, int64_t, const SegTable&, const ExtKV&,
                             const CallerIo&, float, hipStream_t) { std::abort(); }
hipError_t launch_append(void*, void*, const void*, const void*, int, int, int64_t, const MoveList&, int, int, int,
                         const RowMap&, int, hipStream_t) { std::abort(); }
hipError_t launch_roll(void*, void*, const void*, const void*, int, int, int64_t, const MoveList&, const NewRanges&,
                       const RowMap&, int, hipStream_t) { std::abort(); }
hipError_t launch_export(const void*, const void*, void*, void*, int, int, int64_t, const SegTable&, const ExtKV&,
                         const RowMap&, int, hipStream_t) { std::abort(); }
hipError_t launch_similarity(const ScaleRef&, const ScaleRef&, int, int, int, int, int, int, int, int, float*, float*,
                             hipStream_t) { std::abort(); }
hipError_t launch_similarity_static(const ScaleRef&, const ScaleRef&, int, int, int, int, int, int, int, int, float*,
                                    hipStream_t) { std::abort(); }
hipError_t launch_density(const void*, const void*, int, int, int, int, int, int64_t, const SegTable&, const ExtKV&,
                          const CallerIo&, float, float*, float*, hipStream_t) { std::abort(); }
hipError_t launch_theta_flag(const float*, int, double, float, int32_t*, hipStream_t) { std::abort(); }
bool attend_density_fused(int) { std::abort(); }
bool attend_owns_unit(int, int) { return true; }
hipError_t launch_attend_density_bf16(const void*, void*, void*, void*, int, int, int, int, int64_t, const SegTable&, const ExtKV&,
                                      const CallerIo&, float, const GroupEnds&, float*, float*, hipStream_t) { std::abort(); }
}  // namespace amskv
extern "C" hipError_t hipMemcpyAsync(void*, const void*, size_t, hipMemcpyKind, hipStream_t) { std::abort(); }
extern "C" hipError_t hipStreamSynchronize(hipStream_t) { std::abort(); }
extern "C" hipError_t hipHostMalloc(void**, size_t, unsigned int) { std::abort(); }
extern "C" hipError_t hipHostFree(void*) { std::abort(); }
extern "C" hipError_t hipEventCreateWithFlags(hipEvent_t*, unsigned) { std::abort(); }
extern "C" hipError_t hipEventDestroy(hipEvent_t) { std::abort(); }
extern "C" hipError_t hipEventRecord(hipEvent_t, hipStream_t) { std::abort(); }
extern "C" hipError_t hipEventSynchronize(hipEvent_t) { std::abort(); }

static int failures = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                            \
    }                                                                        \
  } while (0)

struct Sched {
  std::vector<int32_t> sides;
};

static void walk_window(const Sched& sc, int32_t layout, int32_t borrow, int32_t fuse) {
  const int n = (int)sc.sides.size();
  std::vector<amskv_layer_policy> pols;
  for (int c = 0; c < 5; ++c)
    for (int w = 0; w < 5; ++w) pols.push_back({c, w, 0});
  pols.push_back({0, 0, 1});
  pols.push_back({2, 1, 1});
  const int L = (int)pols.size(), B = 2, H = 3, D = 64;
  amskv_schedule s{n, sc.sides.data(), sc.sides.data(), B, AMSKV_DTYPE_BF16};
  amskv_policy p{L, pols.data(), 0.f, layout, borrow, fuse, AMSKV_MODE_SCALE_WINDOW, nullptr};
  uint64_t need = 0;
  CHECK(amskv_cache_required_bytes(L, H, D, &s, &p, &need) == AMSKV_OK && need > 0);
  amskv_cache* h = nullptr;
  CHECK(amskv_cache_create(L, H, D, &s, &p, nullptr, 0, &h) == AMSKV_OK && h);
  if (!h) return;
  for (int step = 0; step < n; ++step)
    for (int l = 0; l < L; ++l) {
      CHECK(amskv_append_scale(h, l, step + 1, nullptr, nullptr, nullptr) != AMSKV_OK);  // out of order / range
      CHECK(amskv_append_scale(h, l, step, nullptr, nullptr, nullptr) == AMSKV_OK);
      int32_t n_seg = 0, scale[AMSKV_MAX_SCALES], len[AMSKV_MAX_SCALES], first[AMSKV_MAX_SCALES];
      int64_t off[AMSKV_MAX_SCALES];
      CHECK(amskv_cache_layout(h, l, &n_seg, scale, off, len) == AMSKV_OK);
      CHECK(n_seg >= 1 && n_seg <= step + 1 && scale[n_seg - 1] == step);
      int64_t tok = 0;
      const int64_t cap = amskv_cache_capacity_tokens(h, l);
      for (int i = 0; i < n_seg; ++i) {
        CHECK(len[i] == sc.sides[scale[i]] * sc.sides[scale[i]]);
        CHECK(i == 0 || scale[i] > scale[i - 1]);
        CHECK(off[i] < 0 || off[i] + len[i] <= cap);
        for (int j = 0; j < i; ++j)
          CHECK(off[i] < 0 || off[j] < 0 || off[i] + len[i] <= off[j] || off[j] + len[j] <= off[i]);
        tok += len[i];
      }
      CHECK(amskv_cache_bytes_held(h, l, 1) == 2 * 2 * (int64_t)B * H * D * tok);
      CHECK(amskv_cache_bytes_held(h, l, 0) == 2 * 2 * (int64_t)B * H * D * (tok - len[n_seg - 1]));
      int32_t n2 = 0;
      CHECK(amskv_cache_segments(h, l, &n2, scale, first, off, len) == AMSKV_OK && n2 == n_seg);
      int32_t n_ev = 0, ev[AMSKV_MAX_SCALES];
      CHECK(amskv_cache_last_evicted(h, l, &n_ev, ev) == AMSKV_OK && n_ev >= 0 && n_ev <= step);
      // device work on a plan-only cache is refused, not attempted
      CHECK(amskv_attend(h, l, step, (const void*)16, (void*)16, nullptr) == AMSKV_ERR_NO_DEVICE_MEMORY);
      CHECK(amskv_cache_export(h, l, (void*)16, (void*)16, nullptr) == AMSKV_ERR_NO_DEVICE_MEMORY);
      float dummy[4];
      const int32_t rc = amskv_interscale_similarity(h, l, step, dummy, nullptr, nullptr, nullptr);
      CHECK(rc == AMSKV_ERR_NO_DEVICE_MEMORY || rc == AMSKV_ERR_EVICTED || rc == AMSKV_ERR_INVALID_ARG);
      CHECK(amskv_cache_settle(h, l, nullptr) == AMSKV_OK);
    }
  CHECK(amskv_cache_set_io_layout(h, AMSKV_IO_TOKEN_MAJOR, H * D, H * D, H * D) == AMSKV_ERR_ORDER);
  CHECK(amskv_cache_reset(h) == AMSKV_OK);
  CHECK(amskv_cache_set_io_layout(h, AMSKV_IO_TOKEN_MAJOR, 3 * H * D, 3 * H * D, H * D) == AMSKV_OK);
  CHECK(amskv_append_scale(h, 0, 0, nullptr, nullptr, nullptr) == AMSKV_OK);
  CHECK(amskv_cache_layout(h, L, nullptr, nullptr, nullptr, nullptr) == AMSKV_ERR_INVALID_ARG);
  amskv_cache_destroy(h);
}

static void walk_budget(const Sched& sc) {
  const int n = (int)sc.sides.size();
  int total = 0;
  for (int x : sc.sides) total += x * x;
  std::vector<amskv_layer_budget> buds;
  const int steps[] = {1, 5, 17, 60, 174, 274, 430, 700};
  for (int c_max : steps)
    for (int c_min : steps)
      for (int c_cds : {0, 1, 5, 30}) {
        if (c_min > c_max || c_cds > c_min) continue;
        buds.push_back({c_min, c_max, c_cds, -2.f});   // the Eq. 3 test never fires
        buds.push_back({c_min, c_max, c_cds, 2.f});    // fires at the first overflow
      }
  const int L = (int)buds.size(), B = 1, H = 2, D = 128;
  amskv_schedule s{n, sc.sides.data(), sc.sides.data(), B, AMSKV_DTYPE_F32};
  amskv_policy p{L, nullptr, 0.25f, AMSKV_LAYOUT_COMPACT, 0, 0, AMSKV_MODE_TOKEN_BUDGET, buds.data()};
  amskv_cache* h = nullptr;
  CHECK(amskv_cache_create(L, H, D, &s, &p, nullptr, 0, &h) == AMSKV_OK && h);
  if (!h) return;
  for (int step = 0; step < n; ++step)
    for (int l = 0; l < L; ++l) {
      CHECK(amskv_append_scale(h, l, step, nullptr, nullptr, nullptr) == AMSKV_OK);
      if ((step + l) % 3 == 0) CHECK(amskv_cache_settle(h, l, nullptr) == AMSKV_OK);   // else the next append rolls
      int32_t n_seg = 0;
      std::vector<int32_t> scale(64), first(64), len(64);
      std::vector<int64_t> off(64);
      CHECK(amskv_cache_segments(h, l, &n_seg, nullptr, nullptr, nullptr, nullptr) == AMSKV_OK && n_seg <= 64);
      CHECK(amskv_cache_segments(h, l, &n_seg, scale.data(), first.data(), off.data(), len.data()) == AMSKV_OK);
      const int64_t bgt = amskv_cache_budget_tokens(h, l);
      CHECK(bgt == buds[l].c_min || bgt == buds[l].c_max);
      int64_t cached = 0;
      for (int i = 0; i < n_seg; ++i) {
        CHECK(first[i] >= 0 && len[i] >= 1 && first[i] + len[i] <= sc.sides[scale[i]] * sc.sides[scale[i]]);
        if (off[i] >= 0) cached += len[i];
      }
      CHECK(cached <= buds[l].c_max && cached <= total);
    }
  amskv_cache_destroy(h);
}

// Token windows (sliding window, sinks + window): one budget per layer, scales larger than it are cut.
static void walk_token_window(const Sched& sc) {
  const int n = (int)sc.sides.size();
  std::vector<amskv_layer_budget> wins;
  for (int w : {1, 5, 17, 60, 170, 700})
    for (int sinks : {0, 1, 5, 30})
      if (sinks <= w) wins.push_back({w, w, sinks, 0.f});
  const int L = (int)wins.size(), B = 2, H = 2, D = 64;
  amskv_schedule s{n, sc.sides.data(), sc.sides.data(), B, AMSKV_DTYPE_BF16};
  amskv_policy p{L, nullptr, 0.f, AMSKV_LAYOUT_COMPACT, 0, 0, AMSKV_MODE_TOKEN_WINDOW, wins.data()};
  amskv_cache* h = nullptr;
  CHECK(amskv_cache_create(L, H, D, &s, &p, nullptr, 0, &h) == AMSKV_OK && h);
  if (!h) return;
  int64_t seen = 0;
  for (int step = 0; step < n; ++step) {
    seen += sc.sides[step] * sc.sides[step];
    for (int l = 0; l < L; ++l) {
      CHECK(amskv_append_scale(h, l, step, nullptr, nullptr, nullptr) == AMSKV_OK);
      if ((step + l) % 2 == 0) CHECK(amskv_cache_settle(h, l, nullptr) == AMSKV_OK);
      // a query finishes the iteration too: afterwards the layer holds min(seen, window) tokens
      const int64_t want = std::min<int64_t>(seen, wins[l].c_max);
      if ((step + l) % 2 == 0) CHECK(amskv_cache_bytes_held(h, l, 1) == 2 * 2 * (int64_t)B * H * D * want);
    }
  }
  amskv_policy two = p;
  amskv_layer_budget uneven{3, 9, 0, 0.f};
  two.n_layers = 1;
  two.budget = &uneven;
  uint64_t need = 0;
  CHECK(amskv_cache_required_bytes(1, H, D, &s, &two, &need) == AMSKV_ERR_INVALID_ARG);  // a window is one budget
  amskv_cache_destroy(h);
}

static void bad_arguments() {
  const int32_t sides[3] = {1, 2, 3};
  amskv_layer_policy pol{1, 1, 0};
  amskv_schedule s{3, sides, sides, 1, AMSKV_DTYPE_BF16};
  amskv_policy p{1, &pol, 0.f, AMSKV_LAYOUT_COMPACT, 0, 0, AMSKV_MODE_SCALE_WINDOW, nullptr};
  amskv_cache* h = nullptr;
  uint64_t need = 0;
  CHECK(amskv_cache_create(1, 2, 96, &s, &p, nullptr, 0, &h) == AMSKV_ERR_INVALID_ARG && !h);       // head dim
  CHECK(amskv_cache_create(2, 2, 64, &s, &p, nullptr, 0, &h) == AMSKV_ERR_INVALID_ARG);            // layer count
  CHECK(amskv_cache_required_bytes(1, 2, 64, &s, &p, nullptr) == AMSKV_ERR_INVALID_ARG);
  CHECK(amskv_cache_required_bytes(1, 2, 64, nullptr, &p, &need) == AMSKV_ERR_INVALID_ARG);
  amskv_schedule big{AMSKV_MAX_SCALES + 1, sides, sides, 1, AMSKV_DTYPE_BF16};
  CHECK(amskv_cache_required_bytes(1, 2, 64, &big, &p, &need) == AMSKV_ERR_INVALID_ARG);
  CHECK(amskv_cache_create(1, 2, 64, &s, &p, (void*)256, 16, &h) == AMSKV_ERR_ARENA_TOO_SMALL);
  CHECK(amskv_cache_create(1, 2, 64, &s, &p, (void*)8, 1 << 30, &h) == AMSKV_ERR_INVALID_ARG);     // alignment
  CHECK(amskv_cache_reset(nullptr) == AMSKV_ERR_INVALID_ARG);
  amskv_cache_destroy(nullptr);
  for (int st = 1; st >= -9; --st) CHECK(amskv_status_string(st) != nullptr);
}

int main() {
  const Sched scheds[] = {{{1, 2, 3, 4, 5, 6, 8, 10, 13, 16}}, {{1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64}},
                          {{1, 2, 3}}, {{2, 2, 5, 3}}, {{7}}};
  for (const Sched& sc : scheds) {
    for (int layout : {AMSKV_LAYOUT_COMPACT, AMSKV_LAYOUT_PLANNED})
      for (int borrow : {0, 1})
        for (int fuse : {0, 1}) walk_window(sc, layout, borrow, fuse);
    walk_budget(sc);
    walk_token_window(sc);
  }
  bad_arguments();
  std::printf("host sanitizer driver: %d check(s) failed\n", failures);
  return failures ? 1 : 0;
}
