// Sanitizer driver for the host layer of libamskv (csrc/amskv_api.cpp): built by tests/test_host_sanitize.py
// with -fsanitize=address,undefined together with amskv_api.cpp, it walks plan-only caches (no device memory)
// through every host-side call of the C ABI -- the scale-window policies and schedules of the host layout
// tests, the token-budget mode (Algorithms 1 and 2 with both outcomes of the Eq. 3 test forced by the
// threshold), the error paths -- and checks structural invariants on the way.  Parity with the oracle is the
// business of tests/test_host_layout.py; this program exists so that an out-of-bounds access, a use after
// free or undefined behaviour in the metadata code stops a test run.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <vector>

#include "amskv_internal.hpp"

static int failures = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                            \
    }                                                                        \
  } while (0)

// ---- the device side is not part of this build.  On plan-only caches the launchers and runtime calls are stubs
// that fail loudly if a host path ever reaches them.  In a dry run (g_dry) they emulate instead, on lists of token
// ids, what the kernels would do to the cache of a one-layer cache whose arena is ordinary host memory: the
// attention launch streams the rows its segment table names and writes back the rows its ExtKV asks for (one row
// at a time, in stream order: a row the plan overwrites before it has been read shows up as a wrong id), the roll
// launch moves and copies, the decision kernel answers g_outcome.  What the host layer then reports as the
// layer's list must be what the emulated cache holds.
static bool g_dry = false;
static int g_outcome = 0;              // the device's answer to the Eq. 3 test
static std::vector<int32_t> g_ids;     // token id at every cache offset, -1: never written
static std::vector<int32_t> g_new;     // ids of the rows of the scale being appended
static std::vector<int32_t> g_seen;    // ids the last attention launch streamed, in order
static int g_attends = 0, g_rolls = 0, g_tests = 0;

static hipError_t dry_attend(int64_t cap, const amskv::SegTable& seg, const amskv::ExtKV& ext) {
  amskv::ExtKV e = ext;
  if (e.alt_if != nullptr && *e.alt_if != 0) {
    e.wb_from = e.alt_from;
    e.wb_delta = e.alt_delta;
    e.wb_head_end = e.alt_head_end;
  }
  ++g_attends;
  g_seen.clear();
  for (int g = 0; g < seg.n; ++g)
    for (int i = 0; i < seg.len[g]; ++i) {
      const int j = seg.virt_start[g] + i;
      int32_t id = -1;
      int64_t at = -1;
      if (j >= seg.ext_start) {
        CHECK(j - seg.ext_start < (int)g_new.size());
        id = g_new[j - seg.ext_start];
      } else {
        at = seg.phys_off[g] + i;
        CHECK(at >= 0 && at < cap);
        id = g_ids[at];
        CHECK(id >= 0);
      }
      g_seen.push_back(id);
      const int to = amskv::write_back_row(e, j, seg.total, seg.ext_start);
      if (to >= 0) {
        CHECK(to < cap && to <= j && (at < 0 || to <= at));
        g_ids[to] = id;
      }
    }
  CHECK((int)g_seen.size() == seg.total);
  return hipSuccess;
}

namespace amskv {
hipError_t launch_attend_bf16(const void*, void*, void*, void*, int, int, int, int64_t cap, const SegTable& seg, const ExtKV& ext,
                              const CallerIo&, float, hipStream_t) {
  if (!g_dry) std::abort();
  return dry_attend(cap, seg, ext);
}
hipError_t launch_attend_f32(const void*, void*, void*, void*, int, int, int, int64_t cap, const SegTable& seg, const ExtKV& ext,
                             const CallerIo&, float, hipStream_t) {
  if (!g_dry) std::abort();
  CHECK(ext.alt_if == nullptr && (ext.wb_from >= seg.ext_start));   // the fp32 kernel writes rows of the new scale only
  return dry_attend(cap, seg, ext);
}
hipError_t launch_append(void*, void*, const void*, const void*, int, int, int64_t, const MoveList&, int, int, int,
                         const RowMap&, int, hipStream_t) { std::abort(); }
hipError_t launch_roll(void*, void*, const void*, const void*, int, int, int64_t cap, const MoveList& mv, const NewRanges& nr,
                       const RowMap&, int, hipStream_t) {
  if (!g_dry) std::abort();
  ++g_rolls;
  for (int m = 0; m < mv.n; ++m) {
    CHECK(mv.dst[m] < mv.src[m] && mv.src[m] + mv.len[m] <= cap);
    for (int i = 0; i < mv.len[m]; ++i) g_ids[mv.dst[m] + i] = g_ids[mv.src[m] + i];
  }
  for (int r = 0; r < nr.n; ++r) {
    CHECK(nr.dst[r] >= 0 && nr.dst[r] + nr.len[r] <= cap && nr.src_first[r] + nr.len[r] <= (int)g_new.size());
    for (int i = 0; i < nr.len[r]; ++i) g_ids[nr.dst[r] + i] = g_new[nr.src_first[r] + i];
  }
  return hipSuccess;
}
hipError_t launch_export(const void*, const void*, void*, void*, int, int, int64_t, const SegTable&, const ExtKV&,
                         const RowMap&, int, hipStream_t) { std::abort(); }
hipError_t launch_similarity(const ScaleRef&, const ScaleRef&, int, int, int, int, int, int, int, int, float*, float*,
                             hipStream_t) {
  if (!g_dry) std::abort();
  return hipSuccess;
}
hipError_t launch_similarity_static(const ScaleRef&, const ScaleRef&, int, int, int, int, int, int, int, int, float*,
                                    hipStream_t) { std::abort(); }
hipError_t launch_density(const void*, const void*, int, int, int, int, int, int64_t, const SegTable&, const ExtKV&,
                          const CallerIo&, float, float*, float*, hipStream_t) { std::abort(); }
hipError_t launch_theta_flag(const float*, int, double, float, int32_t* flag, int32_t* flag_host, hipStream_t) {
  if (!g_dry) std::abort();
  ++g_tests;
  *flag = g_outcome;
  *flag_host = g_outcome;
  return hipSuccess;
}
bool attend_density_fused(int) { std::abort(); }
bool attend_owns_unit(int head_dim, int t_q) { return t_q <= (head_dim == 64 ? 256 : 128); }
hipError_t launch_attend_density_bf16(const void*, void*, void*, void*, int, int, int, int, int64_t, const SegTable&, const ExtKV&,
                                      const CallerIo&, float, const GroupEnds&, float*, float*, hipStream_t) { std::abort(); }
}  // namespace amskv
extern "C" hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t) {
  if (!g_dry) std::abort();
  std::memcpy(dst, src, n);
  return hipSuccess;
}
extern "C" hipError_t hipStreamSynchronize(hipStream_t) { std::abort(); }
extern "C" hipError_t hipHostMalloc(void** p, size_t n, unsigned int) {
  if (!g_dry) std::abort();
  *p = std::calloc(1, n);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
extern "C" hipError_t hipHostFree(void* p) {
  if (!g_dry) std::abort();
  std::free(p);
  return hipSuccess;
}
extern "C" hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
  if (!g_dry) std::abort();
  *e = reinterpret_cast<hipEvent_t>(std::malloc(1));
  return hipSuccess;
}
extern "C" hipError_t hipEventDestroy(hipEvent_t e) {
  if (!g_dry) std::abort();
  std::free(e);
  return hipSuccess;
}
extern "C" hipError_t hipEventRecord(hipEvent_t, hipStream_t) {
  if (!g_dry) std::abort();
  return hipSuccess;
}
extern "C" hipError_t hipEventSynchronize(hipEvent_t) {
  if (!g_dry) std::abort();
  return hipSuccess;
}

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

// Dry runs of the token modes through amskv_attend: the plan the attention launch is handed (ExtKV) must leave the
// emulated cache exactly as the host's list says, whichever way the iteration is performed (by the launch, by a
// roll launch of the next call, with the Eq. 3 test answered either way on the "device"), and the launch must
// stream exactly the list as it was before the step followed by the new scale.
static void dry_token_modes(const Sched& sc, int32_t dtype) {
  const int n = (int)sc.sides.size();
  std::vector<int32_t> start(n + 1, 0);
  for (int i = 0; i < n; ++i) start[i + 1] = start[i] + sc.sides[i] * sc.sides[i];
  struct Case { amskv_layer_budget b; int32_t mode; };
  std::vector<Case> cases;
  const int steps[] = {1, 5, 17, 60, 174, 274, 700};
  for (int c_max : steps)
    for (int c_min : steps)
      for (int c_cds : {0, 1, 5, 30}) {
        if (c_min > c_max || c_cds > c_min) continue;
        cases.push_back({{c_min, c_max, c_cds, 0.5f}, AMSKV_MODE_TOKEN_BUDGET});
        if (c_min == c_max) cases.push_back({{c_min, c_max, c_cds, 0.f}, AMSKV_MODE_TOKEN_WINDOW});
      }
  const int B = 1, H = 1, D = 64;
  g_dry = true;
  int variant = 0;
  for (const Case& cs : cases)
    for (int outcome = 0; outcome < 2; ++outcome, ++variant) {
      amskv_schedule s{n, sc.sides.data(), sc.sides.data(), B, dtype};
      amskv_policy p{1, nullptr, 0.f, AMSKV_LAYOUT_COMPACT, 0, 0, cs.mode, &cs.b};
      uint64_t need = 0;
      CHECK(amskv_cache_required_bytes(1, H, D, &s, &p, &need) == AMSKV_OK);
      void* arena = std::aligned_alloc(256, (need + 255) / 256 * 256);
      amskv_cache* h = nullptr;
      CHECK(amskv_cache_create(1, H, D, &s, &p, arena, need, &h) == AMSKV_OK && h);
      if (!h) {
        std::free(arena);
        continue;
      }
      g_outcome = outcome;
      const int64_t cap = amskv_cache_capacity_tokens(h, 0);
      g_ids.assign((size_t)std::max<int64_t>(cap, 1), -1);
      char* fake = reinterpret_cast<char*>(arena);   // any aligned non-null address: the stubs never follow it
      for (int step = 0; step < n; ++step) {
        // (an iteration left over from the step before runs inside this append and copies from that step's scale)
        CHECK(amskv_append_scale(h, 0, step, fake, fake, nullptr) == AMSKV_OK);
        g_new.resize((size_t)(start[step + 1] - start[step]));
        for (size_t i = 0; i < g_new.size(); ++i) g_new[i] = start[step] + (int32_t)i;
        int32_t n_seg = 0;
        std::vector<int32_t> scale(64), first(64), len(64);
        std::vector<int64_t> off(64);
        CHECK(amskv_cache_segments(h, 0, &n_seg, scale.data(), first.data(), off.data(), len.data()) == AMSKV_OK);
        std::vector<int32_t> before;
        for (int i = 0; i < n_seg; ++i)
          for (int k = 0; k < len[i]; ++k) before.push_back(start[scale[i]] + first[i] + k);
        const bool attend = (step + variant) % 4 != 0;   // now and then the step's attention never comes
        if (attend) {
          CHECK(amskv_attend(h, 0, step, fake, fake, nullptr) == AMSKV_OK);
          CHECK(g_seen == before);
        }
        CHECK(amskv_cache_segments(h, 0, &n_seg, scale.data(), first.data(), off.data(), len.data()) == AMSKV_OK);
        int64_t at = 0;
        for (int i = 0; i < n_seg; ++i) {
          if (off[i] < 0) {   // the new scale, still read in place: its iteration waits for the next append
            CHECK(!attend && i == n_seg - 1);
            continue;
          }
          CHECK(off[i] == at);   // one run from offset 0
          for (int k = 0; k < len[i]; ++k) CHECK(g_ids[(size_t)(off[i] + k)] == start[scale[i]] + first[i] + k);
          at += len[i];
        }
        CHECK(at <= amskv_cache_budget_tokens(h, 0) && at <= cap);
      }
      amskv_cache_destroy(h);
      std::free(arena);
    }
  g_dry = false;
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
    dry_token_modes(sc, AMSKV_DTYPE_BF16);
    dry_token_modes(sc, AMSKV_DTYPE_F32);
  }
  bad_arguments();
  CHECK(g_attends > 1000 && g_rolls > 100 && g_tests > 100);   // the dry runs did reach all three kinds of launch
  std::printf("host sanitizer driver: %d check(s) failed (%d attention launches, %d roll launches, %d tests emulated)\n", failures,
              g_attends, g_rolls, g_tests);
  return failures ? 1 : 0;
}
