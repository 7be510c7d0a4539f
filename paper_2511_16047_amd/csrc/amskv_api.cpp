// Host layer of libamskv: schedule, per-layer policy -> kept set, arena layout, segment
// tables, status codes, and the C ABI declared in amskv.h.  All policy decisions are made
// here on the host; the kernels only see token offsets.
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "amskv_internal.hpp"

namespace {

using amskv::CallerIo;
using amskv::ExtKV;
using amskv::MoveList;
using amskv::RowMap;
using amskv::ScaleRef;
using amskv::SegTable;

struct Segment {
  int32_t scale;
  int32_t off;  // token offset inside the layer's [cap] axis; -1: borrowed (read in place)
  int32_t len;
  int32_t first = 0;  // first token of the scale held here (token-budget mode keeps scales in part)
  const void* ext_k = nullptr;  // the caller's K/V of that scale while it is read in place
  const void* ext_v = nullptr;
  bool pending = false;         // fuse_append: slot reserved at `off`, data still only in ext_k/ext_v
};

struct LayerState {
  amskv_layer_policy pol;
  int64_t cap = 0;         // tokens
  uint64_t k_off = 0;      // byte offset of the K region inside the arena
  uint64_t v_off = 0;
  int32_t last_scale = -1;
  std::vector<Segment> segs;        // ascending scale id
  std::vector<int32_t> last_evicted;
  int32_t planned_off[AMSKV_MAX_SCALES];  // PLANNED layout: fixed slot of every scale
  // token-budget mode (Algorithm 1): budgets, the budget in force, and whether the newest scale
  // (last segment, read in place) still awaits its iteration of the algorithm
  // similarity results waiting in the layer's device slot: scale they belong to (-1: none), whether V was included
  int32_t sim_scale = -1;
  bool sim_has_v = false;
  amskv_layer_budget bud = {0, 0, 0, 0.f};
  int32_t c_bgt = 0;
  bool roll_pending = false;
  // amskv_attend leaves the iteration to the next call that needs the layer's state (`deferred`); if the
  // iteration needs the Eq. 3 score, the test has been enqueued and its sums are on their way to the host
  bool deferred = false;
  bool test_pending = false;
  bool device_done = false;  // the deferred iteration's device side was done by the step's attention launch
  hipEvent_t test_done = nullptr;
  hipStream_t test_stream = nullptr;
};

}  // namespace

struct amskv_cache {
  int32_t layers, heads, head_dim, batch, dtype, n_scales, layout, borrow, fuse, mode;
  bool cut_oversize = false;  // token-window mode: a scale larger than the budget keeps its newest tokens instead of being skipped
  int32_t side_h[AMSKV_MAX_SCALES], side_w[AMSKV_MAX_SCALES], tokens[AMSKV_MAX_SCALES];
  float softmax_scale;
  int32_t elem_bytes;
  char* arena = nullptr;
  uint64_t arena_bytes = 0;
  uint64_t ws_off = 0;    // similarity workspace
  uint64_t dens_off = 0;  // attention-density workspace
  int32_t io_layout = AMSKV_IO_HEAD_MAJOR;
  int64_t q_tok = 0, kv_tok = 0, o_tok = 0;  // token strides in elements (token-major tensors only)
  float* theta_host = nullptr;  // token-budget mode: pinned; behind [layers][heads * 4] floats, one decision word per layer
  std::vector<LayerState> layer;
};

namespace {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Section 4.1 taxonomy / Section 4.3 rolling rule in scale units: after scale s arrives the
// layer holds the first n_condensed scales, the `window` scales before s, and s.
inline bool resident(const amskv_layer_policy& p, int s, int k) {
  if (k > s) return false;
  if (p.keep_all) return true;
  return k < p.n_condensed || s - k <= p.window;
}

inline int last_step_resident(const amskv_layer_policy& p, int k, int n_scales) {
  if (p.keep_all || k < p.n_condensed) return n_scales - 1;
  return std::min(n_scales - 1, k + p.window);
}

// Algorithm 1 stores a scale only when a later step will read it.  With borrow_unretained a
// scale that no step after its own reads (the last scale of the schedule; every scale under a
// zero window outside the condensed set) is never copied into the arena.
inline bool stored(const amskv_layer_policy& p, int k, int n_scales, bool borrow) {
  return !borrow || last_step_resident(p, k, n_scales) > k;
}

int validate(int32_t layers, int32_t heads, int32_t head_dim, const amskv_schedule* sc,
             const amskv_policy* po) {
  if (!sc || !po || layers < 1 || heads < 1) return AMSKV_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return AMSKV_ERR_INVALID_ARG;
  if (sc->n_scales < 1 || sc->n_scales > AMSKV_MAX_SCALES || !sc->side_h || !sc->side_w)
    return AMSKV_ERR_INVALID_ARG;
  if (sc->batch < 1) return AMSKV_ERR_INVALID_ARG;
  if (sc->dtype != AMSKV_DTYPE_F32 && sc->dtype != AMSKV_DTYPE_BF16) return AMSKV_ERR_INVALID_ARG;
  int64_t total = 0;
  for (int i = 0; i < sc->n_scales; ++i) {
    if (sc->side_h[i] < 1 || sc->side_w[i] < 1) return AMSKV_ERR_INVALID_ARG;
    int64_t t = (int64_t)sc->side_h[i] * sc->side_w[i];
    if (t > (1 << 20)) return AMSKV_ERR_INVALID_ARG;
    total += t;
  }
  if (total > (1 << 22)) return AMSKV_ERR_INVALID_ARG;
  if ((int64_t)sc->batch * heads > (1 << 24)) return AMSKV_ERR_INVALID_ARG;
  // launch grids count (b, h, block of >= 32 query rows) units and 16-byte chunks of a scale in 32 bits
  for (int i = 0; i < sc->n_scales; ++i) {
    const int64_t t = (int64_t)sc->side_h[i] * sc->side_w[i];
    if ((int64_t)sc->batch * heads * ((t + 31) / 32) > (1 << 30)) return AMSKV_ERR_INVALID_ARG;
    if ((int64_t)sc->batch * heads * t * (head_dim / 4) > ((int64_t)1 << 39)) return AMSKV_ERR_INVALID_ARG;
  }
  if (po->n_layers != layers) return AMSKV_ERR_INVALID_ARG;
  if (po->layout != AMSKV_LAYOUT_COMPACT && po->layout != AMSKV_LAYOUT_PLANNED)
    return AMSKV_ERR_INVALID_ARG;
  if (po->borrow_unretained != 0 && po->borrow_unretained != 1) return AMSKV_ERR_INVALID_ARG;
  if (po->fuse_append != 0 && po->fuse_append != 1) return AMSKV_ERR_INVALID_ARG;
  if (!(po->softmax_scale >= 0.f) || !std::isfinite(po->softmax_scale)) return AMSKV_ERR_INVALID_ARG;
  if (po->mode == AMSKV_MODE_TOKEN_BUDGET || po->mode == AMSKV_MODE_TOKEN_WINDOW) {
    if (!po->budget || po->layout != AMSKV_LAYOUT_COMPACT || po->borrow_unretained || po->fuse_append)
      return AMSKV_ERR_INVALID_ARG;
    for (int l = 0; l < layers; ++l) {
      const amskv_layer_budget& b = po->budget[l];
      if (b.c_cds < 0 || b.c_min < b.c_cds || b.c_max < b.c_min || b.c_max < 1 || b.c_max > (1 << 22) ||
          std::isnan(b.theta))
        return AMSKV_ERR_INVALID_ARG;
      if (po->mode == AMSKV_MODE_TOKEN_WINDOW && b.c_min != b.c_max) return AMSKV_ERR_INVALID_ARG;  // one fixed window
    }
    return AMSKV_OK;
  }
  if (po->mode != AMSKV_MODE_SCALE_WINDOW || !po->layer) return AMSKV_ERR_INVALID_ARG;
  for (int l = 0; l < layers; ++l)
    if (po->layer[l].n_condensed < 0 || po->layer[l].window < 0) return AMSKV_ERR_INVALID_ARG;
  return AMSKV_OK;
}

// Capacity of a layer in the COMPACT layout: the largest stored-token count over all steps.
int64_t compact_capacity(const amskv_layer_policy& p, const int32_t* tokens, int n_scales, bool borrow) {
  int64_t best = 0;
  for (int s = 0; s < n_scales; ++s) {
    int64_t sum = 0;
    for (int k = 0; k <= s; ++k)
      if (resident(p, s, k) && stored(p, k, n_scales, borrow)) sum += tokens[k];
    best = std::max(best, sum);
  }
  return best;
}

// PLANNED layout: the schedule and the policy fix, at create time, the interval of steps
// [k, last_k] during which scale k is resident.  Give every stored scale a slot such that
// scales with overlapping lifetimes never overlap in memory, so eviction needs no data movement
// at all.  plan_slots returns the capacity reached.
// One first-fit placement: the stored scales are taken in `order`, each at the lowest offset that is free over its
// whole residency interval.
int64_t place_slots(const amskv_layer_policy& p, const int32_t* tokens, int n_scales, const std::vector<int>& order,
                    int32_t* off_out) {
  for (int i = 0; i < n_scales; ++i) off_out[i] = -1;
  std::vector<char> placed(n_scales, 0);
  int64_t cap = 0;
  for (int k : order) {
    const int lo = k, hi = last_step_resident(p, k, n_scales);
    std::vector<std::pair<int64_t, int64_t>> busy;
    for (int j = 0; j < n_scales; ++j) {
      if (!placed[j]) continue;
      const int jl = j, jh = last_step_resident(p, j, n_scales);
      if (jl <= hi && lo <= jh) busy.emplace_back(off_out[j], (int64_t)off_out[j] + tokens[j]);
    }
    std::sort(busy.begin(), busy.end());
    int64_t at = 0;
    for (auto& iv : busy) {
      if (iv.first - at >= tokens[k]) break;
      at = std::max(at, iv.second);
    }
    off_out[k] = (int32_t)at;
    placed[k] = 1;
    cap = std::max(cap, at + tokens[k]);
  }
  return cap;
}

// How broken up the kept scales are under a placement: over all steps, the number of physically separate runs
// the queries of the step stream (kept scales in ascending order, neighbours merged when they touch), weighted by
// the step's query count.
int64_t placement_cost(const amskv_layer_policy& p, const int32_t* tokens, int n_scales, const int32_t* off) {
  int64_t cost = 0;
  for (int s = 0; s < n_scales; ++s) {
    int runs = 0;
    int64_t end = -1;
    for (int k = 0; k <= s; ++k) {
      if (!resident(p, s, k)) continue;
      if (off[k] < 0 || off[k] != end) ++runs;  // a scale read in place is a run of its own
      end = off[k] < 0 ? -1 : (int64_t)off[k] + tokens[k];
    }
    cost += (int64_t)runs * tokens[s];
  }
  return cost;
}

int64_t plan_slots(const amskv_layer_policy& p, const int32_t* tokens, int n_scales, bool borrow,
                   int32_t* off_out) {
  std::vector<int> stored_scales;
  for (int i = 0; i < n_scales; ++i)
    if (stored(p, i, n_scales, borrow)) stored_scales.push_back(i);
  // Candidate orders for the first-fit placement.  Largest first packs windows of unequal scales tightest.
  // Ascending puts scales back to back wherever lifetimes allow (a layer that keeps everything becomes one
  // contiguous run per (b,h)).  Condensed scales first, then the others by descending last step, makes the scales
  // that the last -- largest -- steps read sit next to each other in reading order.  The smallest capacity wins;
  // among equals, the placement whose steps stream the fewest separate runs (one table entry and one long burst
  // per run).
  std::vector<std::vector<int>> orders(3, stored_scales);
  std::stable_sort(orders[0].begin(), orders[0].end(), [&](int a, int b) { return tokens[a] > tokens[b]; });
  std::stable_sort(orders[2].begin(), orders[2].end(), [&](int a, int b) {
    const bool ca = a < p.n_condensed || p.keep_all, cb = b < p.n_condensed || p.keep_all;
    if (ca != cb) return ca;
    if (ca) return a < b;
    return last_step_resident(p, a, n_scales) > last_step_resident(p, b, n_scales);
  });
  int64_t best_cap = -1, best_cost = 0;
  for (const std::vector<int>& order : orders) {
    int32_t off[AMSKV_MAX_SCALES];
    const int64_t cap = place_slots(p, tokens, n_scales, order, off);
    const int64_t cost = placement_cost(p, tokens, n_scales, off);
    if (best_cap < 0 || cap < best_cap || (cap == best_cap && cost < best_cost)) {
      best_cap = cap;
      best_cost = cost;
      std::copy(off, off + n_scales, off_out);
    }
  }
  return best_cap;
}

struct Plan {
  std::vector<int64_t> cap;
  std::vector<uint64_t> k_off, v_off;
  std::vector<std::vector<int32_t>> slot;
  uint64_t ws_off = 0, dens_off = 0, total = 0;
};

void build_plan(int32_t layers, int32_t heads, int32_t head_dim, const amskv_schedule* sc,
                const amskv_policy* po, Plan* pl) {
  int32_t tokens[AMSKV_MAX_SCALES];
  for (int i = 0; i < sc->n_scales; ++i) tokens[i] = sc->side_h[i] * sc->side_w[i];
  const uint64_t eb = sc->dtype == AMSKV_DTYPE_BF16 ? 2 : 4;
  const uint64_t row = (uint64_t)head_dim * eb;
  const uint64_t bh = (uint64_t)sc->batch * heads;
  const bool borrow = po->borrow_unretained != 0;
  uint64_t at = 0;
  pl->cap.resize(layers);
  pl->k_off.resize(layers);
  pl->v_off.resize(layers);
  pl->slot.assign(layers, std::vector<int32_t>(AMSKV_MAX_SCALES, 0));
  for (int l = 0; l < layers; ++l) {
    int64_t cap;
    if (po->mode != AMSKV_MODE_SCALE_WINDOW)
      cap = po->budget[l].c_max;  // Section 4.3: C_max is the most a layer ever holds
    else if (po->layout == AMSKV_LAYOUT_PLANNED)
      cap = plan_slots(po->layer[l], tokens, sc->n_scales, borrow, pl->slot[l].data());
    else
      cap = compact_capacity(po->layer[l], tokens, sc->n_scales, borrow);
    pl->cap[l] = cap;
    pl->k_off[l] = at;
    at = align_up(at + bh * (uint64_t)cap * row);
    pl->v_off[l] = at;
    at = align_up(at + bh * (uint64_t)cap * row);
  }
  pl->ws_off = at;
  // similarity workspace: per (tensor, b, h) four partial sums, then per (layer, tensor, h) four totals
  // (and one word per layer for the outcome of Algorithm 1's test when it is decided on the device)
  at = align_up(at + (2 * bh * 4 + (uint64_t)layers * 2 * heads * 4 + (uint64_t)layers) * sizeof(float));
  // attention-density workspace: per (b, h, block of 32 query rows) one partial sum per group of keys,
  // then per head one total per group
  int32_t t_max = 0;
  for (int i = 0; i < sc->n_scales; ++i) t_max = std::max(t_max, tokens[i]);
  pl->dens_off = at;
  at = align_up(at + (bh * (uint64_t)((t_max + 31) / 32) + (uint64_t)heads) * AMSKV_MAX_SCALES * sizeof(float));
  pl->total = at;
}

// Rows of a tensor of the caller's that holds t tokens per (b,h): head-major [B][H][t][D], or
// token-major [B][t][..] with `tok_stride` elements from one token to the next.
inline RowMap caller_map(const amskv_cache* c, int64_t t, int64_t tok_stride) {
  const int64_t row = (int64_t)c->head_dim * c->elem_bytes;
  if (c->io_layout == AMSKV_IO_HEAD_MAJOR) return RowMap{c->heads * t * row, t * row, row};
  return RowMap{t * tok_stride * c->elem_bytes, row, tok_stride * c->elem_bytes};
}

// Rows of a layer's K (or V) region: [B][H][cap][D].
inline RowMap arena_map(const amskv_cache* c, const LayerState& L) {
  const int64_t row = (int64_t)c->head_dim * c->elem_bytes;
  return RowMap{c->heads * L.cap * row, L.cap * row, row};
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

inline bool bad_layer(const amskv_cache* c, int32_t layer) {
  return !c || layer < 0 || layer >= c->layers;
}

// Segment table for the kernels; a borrowed segment (always the newest scale, hence last)
// becomes the external tail of the virtual concatenation.
SegTable seg_table(const LayerState& L, ExtKV* ext, bool merge = true) {
  SegTable t;
  std::memset(&t, 0, sizeof(t));
  ext->k = ext->v = nullptr;
  ext->wb_from = ext->alt_from = amskv::kNoWriteBack;
  ext->wb_delta = ext->alt_delta = 0;
  ext->wb_head_end = ext->alt_head_end = 0;
  ext->alt_if = nullptr;
  int32_t v = 0;
  int32_t ext_start = -1;
  int n = 0;
  for (const Segment& g : L.segs) {
    const bool outside = g.off < 0 || g.pending;
    // neighbours that are also back to back in memory form one run for the kernels (in the
    // COMPACT layout the whole cached part is one run; token-budget mode relies on that to
    // stay within the table however many partial scales it holds)
    if (merge && !outside && n > 0 && ext_start < 0 && t.phys_off[n - 1] + t.len[n - 1] == g.off) {
      t.len[n - 1] += g.len;
    } else {
      t.virt_start[n] = v;
      t.phys_off[n] = g.off < 0 ? 0 : g.off;
      t.len[n] = g.len;
      ++n;
    }
    if (outside) {
      ext_start = v;
      ext->k = g.ext_k;
      ext->v = g.ext_v;
    }
    v += g.len;
  }
  t.n = n;
  t.total = v;
  t.ext_start = ext_start < 0 ? v : ext_start;
  return t;
}

inline bool whole_scale(const amskv_cache* c, const Segment& g, int s) {
  return g.scale == s && g.first == 0 && g.len == c->tokens[s];
}

inline float* similarity_slot(const amskv_cache* c, int layer) {
  float* partial = (float*)(c->arena + c->ws_off);
  return partial + 2 * (uint64_t)c->batch * c->heads * 4 + (uint64_t)layer * 2 * c->heads * 4;
}

// Where the device leaves the outcome of a layer's Eq. 3 test (behind the slots of all layers), and where the
// host finds its copy (behind the sums of all layers in the pinned block).
inline int32_t* theta_flag_dev(const amskv_cache* c, int layer) { return (int32_t*)similarity_slot(c, c->layers) + layer; }
inline int32_t* theta_flag_host(const amskv_cache* c, int layer) {
  return (int32_t*)(c->theta_host + (size_t)c->layers * c->heads * 4) + layer;
}

// Eq. 3 between scale s (segment cur) and the upsampled scale s-1 (segment prev), both held
// whole: enqueue the kernels that leave, in the layer's result slot, per head four sums (cosine
// total, k.k^, |k|^2, |k^|^2) of K at [0 .. 4H) and, when want_v, of V at [4H .. 8H).
// Where a whole scale sits: in the caller's tensors while it is read in place, else in the layer's regions.
ScaleRef scale_ref(const amskv_cache* c, const LayerState& L, const Segment& g, bool want_v) {
  ScaleRef r;
  if (g.off < 0 || g.pending) {
    r.k = g.ext_k;
    r.v = want_v ? g.ext_v : nullptr;
    r.map = caller_map(c, g.len, c->kv_tok);
    r.off_tokens = 0;
  } else {
    r.k = c->arena + L.k_off;
    r.v = want_v ? c->arena + L.v_off : nullptr;
    r.map = arena_map(c, L);
    r.off_tokens = g.off;
  }
  return r;
}

int similarity_launch(amskv_cache* c, LayerState& L, int layer, const Segment& cur, const Segment& prev, int s,
                      bool want_v, hipStream_t st) {
  auto ref = [&](const Segment& g) { return scale_ref(c, L, g, want_v); };
  hipError_t e = amskv::launch_similarity(ref(cur), ref(prev), c->batch, c->heads, c->head_dim, c->dtype,
                                          c->side_h[s], c->side_w[s], c->side_h[s - 1], c->side_w[s - 1],
                                          (float*)(c->arena + c->ws_off), similarity_slot(c, layer), st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  L.sim_scale = s;
  L.sim_has_v = want_v;
  return AMSKV_OK;
}

// The same, then the sums brought to host[0 .. 8H).  Waits for the stream.
int similarity_sums(amskv_cache* c, LayerState& L, int layer, const Segment& cur, const Segment& prev, int s,
                    bool want_v, std::vector<float>* host, hipStream_t st) {
  int rc = similarity_launch(c, L, layer, cur, prev, s, want_v, st);
  if (rc) return rc;
  host->assign(2 * (size_t)c->heads * 4, 0.f);
  const size_t n_t = want_v ? 2 : 1;
  hipError_t e = hipMemcpyAsync(host->data(), similarity_slot(c, layer), n_t * c->heads * 4 * sizeof(float),
                                hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  e = hipStreamSynchronize(st);
  return e == hipSuccess ? AMSKV_OK : AMSKV_ERR_HIP;
}

// Algorithm 1's test for a cache-demanding layer: Eq. 3 (cosine form, mean over heads) of the
// newest scale against the scale before it, compared with theta.  Either the outcome is known
// without device work (kTestFails, kTestHolds), or the kernels -- the last of which leaves the decision
// word in the layer's pinned slot -- and an event behind them are enqueued (kTestEnqueued).
enum { kTestFails = 0, kTestHolds = 1, kTestEnqueued = 2 };
int start_theta_test(amskv_cache* c, LayerState& L, const Segment& cur, hipStream_t st, int* state) {
  *state = kTestFails;
  if (L.bud.theta > 1.f) {
    *state = kTestHolds;
    return AMSKV_OK;
  }
  if (L.bud.theta < -1.f || cur.scale < 1) return AMSKV_OK;
  const Segment* prev = nullptr;
  for (const Segment& g : L.segs)
    if (&g != &L.segs.back() && whole_scale(c, g, cur.scale - 1)) prev = &g;
  if (!prev) return AMSKV_OK;  // the earlier scale is not cached whole: no score, no expansion
  if (!c->arena || !cur.ext_k || !c->theta_host || !L.test_done) return AMSKV_ERR_NO_DEVICE_MEMORY;
  const int layer = (int)(&L - c->layer.data());
  int rc = similarity_launch(c, L, layer, cur, *prev, cur.scale, false, st);
  if (rc) return rc;
  // the decision is taken on the device (so that a launch behind it can act on it); the same kernel leaves the word
  // in pinned host memory, where the host reads it behind the event
  if (amskv::launch_theta_flag(similarity_slot(c, layer), c->heads, (double)c->batch * c->tokens[cur.scale], L.bud.theta,
                               theta_flag_dev(c, layer), theta_flag_host(c, layer), st) != hipSuccess)
    return AMSKV_ERR_HIP;
  if (hipEventRecord(L.test_done, st) != hipSuccess) return AMSKV_ERR_HIP;
  L.test_stream = st;
  *state = kTestEnqueued;
  return AMSKV_OK;
}

// Waits for the enqueued test of the layer (only for it, not for the stream) and compares.
int read_theta_test(amskv_cache* c, LayerState& L, bool* below) {
  if (hipEventSynchronize(L.test_done) != hipSuccess) return AMSKV_ERR_HIP;
  const int layer = (int)(&L - c->layer.data());
  *below = *theta_flag_host(c, layer) != 0;
  return AMSKV_OK;
}

// Token-budget mode: Algorithm 1's iteration for the newest scale, which until now has been read
// in place as the last segment.  Decides whether the scale is cached at all, expands the budget
// if the layer tests as cache-demanding (the test is made at every iteration that overflows the
// budget while it still is c_min), and applies Algorithm 2 to the token list (cached tokens
// followed by the new scale): the first c_cds tokens and the last (budget - c_cds) tokens stay.
// Survivors slide toward offset 0 and what stays of the new scale is copied behind them, in one launch.
// on_device != kRollNone: the attention kernel of this step has already done the device side of the iteration --
// written the whole scale behind the cached tokens (kRollAppended: the scale fits the budget without trimming), or
// moved the survivors and written what stays of the scale (kRollTrimmed: the outcome was known before the step:
// no Eq. 3 test due, one owner per unit), or done whichever of the two the Eq. 3 test, decided on the device just
// before the launch, called for (kRollEitherWay: the host learns the outcome later, so its part is deferred and
// waits for the test's event) -- so only the host's list is left to update.
// may_defer (amskv_attend): leave the iteration to the next call on the layer; if it needs the Eq. 3 score from
// the device, enqueue the test now, so that the later call finds the result waiting.  An iteration that is never
// asked for (a reset comes first, as after the last step of an image) costs no device work.
enum { kRollNone = 0, kRollAppended = 1, kRollTrimmed = 2, kRollEitherWay = 3 };
int roll_budget(amskv_cache* c, LayerState& L, hipStream_t st, int on_device = kRollNone, bool may_defer = false) {
  if (!L.roll_pending) return AMSKV_OK;
  const Segment cur = L.segs.back();
  const int32_t t_new = cur.len;
  int64_t n_old = 0;
  for (size_t i = 0; i + 1 < L.segs.size(); ++i) n_old += L.segs[i].len;
  int32_t bgt = L.c_bgt;
  bool cache_it = c->cut_oversize || t_new <= L.bud.c_max;
  const bool overflow = cache_it && n_old + t_new > bgt;
  const bool wants_test = overflow && bgt == L.bud.c_min && L.bud.c_max > L.bud.c_min;
  if (L.deferred) {
    // the part amskv_attend left: same state as then; what is enqueued goes behind that step's own work
    st = L.test_stream;
    L.deferred = false;
    if (L.device_done) on_device = kRollEitherWay;
    L.device_done = false;
  } else if (may_defer && on_device == kRollEitherWay) {
    L.deferred = true;  // test_pending was set by the caller, which enqueued the test in front of its launch
    L.device_done = true;
    L.test_stream = st;
    return AMSKV_OK;
  } else if (may_defer && on_device == kRollNone) {
    if (wants_test) {
      int state = kTestFails;
      int rc = start_theta_test(c, L, cur, st, &state);
      if (rc) return rc;
      L.test_pending = state == kTestEnqueued;
    }
    L.deferred = true;
    L.test_stream = st;
    return AMSKV_OK;
  }
  if (overflow) {
    if (wants_test) {
      int state = kTestFails;
      if (!L.test_pending) {
        int rc = start_theta_test(c, L, cur, st, &state);
        if (rc) return rc;
      }
      if (L.test_pending || state == kTestEnqueued) {
        bool below = false;
        int rc = read_theta_test(c, L, &below);
        if (rc) return rc;
        L.test_pending = false;
        state = below ? kTestHolds : kTestFails;
      }
      if (state == kTestHolds) bgt = L.bud.c_max;
    }
    if (t_new > bgt && !c->cut_oversize) cache_it = false;
  }

  struct CopyRange {
    int32_t src_first, len, dst;
  };
  std::vector<Segment> next;
  std::vector<int32_t> evicted;
  std::vector<CopyRange> copies;
  MoveList mv;
  std::memset(&mv, 0, sizeof(mv));
  if (!cache_it) {
    next.assign(L.segs.begin(), L.segs.end() - 1);
  } else {
    const int64_t total = n_old + t_new;
    const bool trim = total > bgt;
    const int64_t head_end = trim ? L.bud.c_cds : total;                       // keep [0, head_end)
    const int64_t tail_begin = trim ? total - (bgt - L.bud.c_cds) : total;     // and [tail_begin, total)
    int64_t pos = 0;
    int32_t at = 0;
    for (size_t i = 0; i < L.segs.size(); ++i) {
      const Segment& g = L.segs[i];
      const bool is_new = i + 1 == L.segs.size();
      const int64_t lo = pos, hi = pos + g.len;
      const int64_t range[2][2] = {{lo, std::min(hi, head_end)}, {std::max(lo, tail_begin), hi}};
      int64_t kept = 0;
      for (int r = 0; r < 2; ++r) {
        const int64_t a = range[r][0], b = range[r][1];
        if (b <= a) continue;
        Segment n;
        n.scale = g.scale;
        n.first = g.first + (int32_t)(a - lo);
        n.len = (int32_t)(b - a);
        n.off = at;
        if (is_new) {
          copies.push_back({n.first, n.len, at});
        } else {
          const int32_t src = g.off + (int32_t)(a - lo);
          if (src != at) {
            if (mv.n > 0 && mv.src[mv.n - 1] + mv.len[mv.n - 1] == src &&
                mv.dst[mv.n - 1] + mv.len[mv.n - 1] == at) {
              mv.len[mv.n - 1] += n.len;
            } else {
              if (mv.n == AMSKV_MAX_SCALES) return AMSKV_ERR_INVALID_ARG;  // cannot happen: survivors form one run
              mv.src[mv.n] = src;
              mv.dst[mv.n] = at;
              mv.len[mv.n] = n.len;
              ++mv.n;
            }
          }
        }
        at += n.len;
        kept += n.len;
        next.push_back(n);
      }
      if (!is_new && kept < g.len && (evicted.empty() || evicted.back() != g.scale)) evicted.push_back(g.scale);
      pos = hi;
    }
    if (at > L.cap) return AMSKV_ERR_ARENA_TOO_SMALL;  // cannot happen: at <= budget <= c_max
  }

  // (cannot fail: the caller derived what the launch writes from the same rule)
  if (on_device == kRollAppended && !(mv.n == 0 && copies.size() == 1 && copies[0].src_first == 0 && copies[0].len == t_new &&
                                      copies[0].dst == (int32_t)n_old))
    return AMSKV_ERR_INVALID_ARG;
  if (c->arena && cur.ext_k && on_device == kRollNone && (mv.n > 0 || !copies.empty())) {
    const int bh = c->batch * c->heads;
    const int row_bytes = c->head_dim * c->elem_bytes;
    amskv::NewRanges nr;
    std::memset(&nr, 0, sizeof(nr));
    for (const CopyRange& r : copies) {  // at most the head and the tail of the new scale
      nr.src_first[nr.n] = r.src_first;
      nr.len[nr.n] = r.len;
      nr.dst[nr.n] = r.dst;
      ++nr.n;
    }
    hipError_t e = amskv::launch_roll(c->arena + L.k_off, c->arena + L.v_off, cur.ext_k, cur.ext_v, bh, row_bytes, L.cap,
                                      mv, nr, caller_map(c, t_new, c->kv_tok), c->heads, st);
    if (e != hipSuccess) return AMSKV_ERR_HIP;
  }
  L.segs.swap(next);
  L.last_evicted.swap(evicted);
  L.c_bgt = bgt;
  L.roll_pending = false;
  return AMSKV_OK;
}

// An iteration of Algorithm 1 whose Eq. 3 test is still on its way is finished before anything reads or changes
// the layer's state (the cache object is never const where it was created; the queries only promise not to
// change what they report).
int finish_iteration(const amskv_cache* cc, int32_t layer) {
  amskv_cache* c = const_cast<amskv_cache*>(cc);
  LayerState& L = c->layer[layer];
  return L.deferred ? roll_budget(c, L, L.test_stream) : AMSKV_OK;
}

// fuse_append: a scale whose attend never came still lives only in the caller's buffers; copy it
int flush_pending(amskv_cache* c, LayerState& L, hipStream_t st) {
  const int bh = c->batch * c->heads;
  const int row_bytes = c->head_dim * c->elem_bytes;
  for (Segment& g : L.segs) {
    if (!g.pending) continue;
    if (g.ext_k) {
      MoveList none;
      std::memset(&none, 0, sizeof(none));
      hipError_t e = amskv::launch_append(c->arena + L.k_off, c->arena + L.v_off, g.ext_k, g.ext_v, bh, row_bytes,
                                          L.cap, none, g.len, g.off, 0, caller_map(c, g.len, c->kv_tok), c->heads, st);
      if (e != hipSuccess) return AMSKV_ERR_HIP;
    }
    g.pending = false;
    g.ext_k = g.ext_v = nullptr;
  }
  return AMSKV_OK;
}

}  // namespace

extern "C" {

const char* amskv_status_string(int32_t st) {
  switch (st) {
    case AMSKV_OK: return "ok";
    case AMSKV_ERR_INVALID_ARG: return "invalid argument";
    case AMSKV_ERR_ORDER: return "call out of order";
    case AMSKV_ERR_EVICTED: return "scale not resident";
    case AMSKV_ERR_ARENA_TOO_SMALL: return "arena too small";
    case AMSKV_ERR_HIP: return "HIP runtime error";
    case AMSKV_ERR_NO_DEVICE_MEMORY: return "plan-only cache has no device memory";
    case AMSKV_ERR_STATIC_LIMIT: return "batch * heads exceeds AMSKV_STATIC_MAX_UNITS, the size of the static workspace";
    case AMSKV_ERR_NO_HOST_MEMORY: return "host memory allocation failed";
    default: return "unknown status";
  }
}

int32_t amskv_cache_required_bytes(int32_t layers, int32_t heads, int32_t head_dim,
                                   const amskv_schedule* sc, const amskv_policy* po,
                                   uint64_t* bytes_out) try {
  if (!bytes_out) return AMSKV_ERR_INVALID_ARG;
  int rc = validate(layers, heads, head_dim, sc, po);
  if (rc) return rc;
  Plan pl;
  build_plan(layers, heads, head_dim, sc, po, &pl);
  *bytes_out = pl.total;
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_create(int32_t layers, int32_t heads, int32_t head_dim,
                           const amskv_schedule* sc, const amskv_policy* po, void* arena_dev,
                           uint64_t arena_bytes, amskv_cache** out) try {
  if (!out) return AMSKV_ERR_INVALID_ARG;
  *out = nullptr;
  int rc = validate(layers, heads, head_dim, sc, po);
  if (rc) return rc;
  Plan pl;
  build_plan(layers, heads, head_dim, sc, po, &pl);
  if (arena_dev) {
    if (((uintptr_t)arena_dev) % kAlign) return AMSKV_ERR_INVALID_ARG;
    if (arena_bytes < pl.total) return AMSKV_ERR_ARENA_TOO_SMALL;
  }
  amskv_cache* c = new (std::nothrow) amskv_cache();
  if (!c) return AMSKV_ERR_NO_HOST_MEMORY;
  struct Owner {  // destroys the half-built cache on every way out but the last
    amskv_cache* c;
    ~Owner() {
      if (c) amskv_cache_destroy(c);
    }
  } owner{c};
  c->layers = layers;
  c->heads = heads;
  c->head_dim = head_dim;
  c->batch = sc->batch;
  c->dtype = sc->dtype;
  c->n_scales = sc->n_scales;
  c->layout = po->layout;
  c->borrow = po->borrow_unretained;
  c->fuse = po->fuse_append;
  // the token window is the token-budget machinery with one fixed budget and oversize scales cut
  c->mode = po->mode == AMSKV_MODE_TOKEN_WINDOW ? AMSKV_MODE_TOKEN_BUDGET : po->mode;
  c->cut_oversize = po->mode == AMSKV_MODE_TOKEN_WINDOW;
  c->elem_bytes = sc->dtype == AMSKV_DTYPE_BF16 ? 2 : 4;
  c->softmax_scale = po->softmax_scale > 0.f ? po->softmax_scale : 1.0f / std::sqrt((float)head_dim);
  for (int i = 0; i < sc->n_scales; ++i) {
    c->side_h[i] = sc->side_h[i];
    c->side_w[i] = sc->side_w[i];
    c->tokens[i] = sc->side_h[i] * sc->side_w[i];
  }
  c->arena = (char*)arena_dev;
  c->arena_bytes = arena_bytes;
  c->ws_off = pl.ws_off;
  c->dens_off = pl.dens_off;
  c->layer.resize(layers);
  for (int l = 0; l < layers; ++l) {
    LayerState& L = c->layer[l];
    if (c->mode == AMSKV_MODE_TOKEN_BUDGET) {
      L.pol = amskv_layer_policy{0, 0, 0};
      L.bud = po->budget[l];
      L.c_bgt = L.bud.c_min;
    } else {
      L.pol = po->layer[l];
    }
    L.cap = pl.cap[l];
    L.k_off = pl.k_off[l];
    L.v_off = pl.v_off[l];
    for (int i = 0; i < AMSKV_MAX_SCALES; ++i) L.planned_off[i] = pl.slot[l][i];
  }
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET && c->arena) {
    // where the Eq. 3 sums of each layer's test arrive, and the event that says they have
    bool ok = hipHostMalloc((void**)&c->theta_host, ((size_t)layers * heads * 4 + layers) * sizeof(float), hipHostMallocDefault) == hipSuccess;
    for (int l = 0; ok && l < layers; ++l)
      ok = hipEventCreateWithFlags(&c->layer[l].test_done, hipEventDisableTiming) == hipSuccess;
    if (!ok) return AMSKV_ERR_HIP;
  }
  owner.c = nullptr;
  *out = c;
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_append_scale(amskv_cache* c, int32_t layer, int32_t s, const void* K_dev,
                           const void* V_dev, void* stream) try {
  if (bad_layer(c, layer) || s < 0 || s >= c->n_scales) return AMSKV_ERR_INVALID_ARG;
  if ((K_dev == nullptr) != (V_dev == nullptr) || misaligned(K_dev) || misaligned(V_dev)) return AMSKV_ERR_INVALID_ARG;
  LayerState& L = c->layer[layer];
  if (s != L.last_scale + 1) return AMSKV_ERR_ORDER;
  if (K_dev && !c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;

  const int bh = c->batch * c->heads;
  const int row_bytes = c->head_dim * c->elem_bytes;
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET) {
    // the previous scale's iteration of Algorithm 1, if its attend never came; then scale s is
    // only recorded: the attention of step s reads it in place, its own iteration follows that
    int rc = roll_budget(c, L, (hipStream_t)stream);
    if (rc) return rc;
    Segment cur;
    cur.scale = s;
    cur.len = c->tokens[s];
    cur.off = -1;
    cur.ext_k = K_dev;
    cur.ext_v = V_dev;
    L.segs.push_back(cur);
    L.roll_pending = true;
    L.last_scale = s;
    return AMSKV_OK;
  }
  int frc = flush_pending(c, L, (hipStream_t)stream);
  if (frc) return frc;

  // new resident list (ascending scale id) and where each segment goes; a borrowed segment of
  // the previous step is by construction not resident any more and simply drops out
  std::vector<Segment> next;
  std::vector<int32_t> evicted;
  MoveList mv;
  std::memset(&mv, 0, sizeof(mv));
  int32_t at = 0;
  for (const Segment& g : L.segs) {
    if (!resident(L.pol, s, g.scale)) {
      evicted.push_back(g.scale);
      continue;
    }
    Segment n = g;
    if (c->layout == AMSKV_LAYOUT_COMPACT) {
      n.off = at;
      if (n.off != g.off) {
        mv.src[mv.n] = g.off;
        mv.dst[mv.n] = n.off;
        mv.len[mv.n] = g.len;
        ++mv.n;
      }
    }
    at += n.len;
    next.push_back(n);
  }
  Segment cur;
  cur.scale = s;
  cur.len = c->tokens[s];
  const bool keep_copy = stored(L.pol, s, c->n_scales, c->borrow != 0);
  if (keep_copy) {
    cur.off = c->layout == AMSKV_LAYOUT_COMPACT ? at : L.planned_off[s];
    if ((int64_t)cur.off + cur.len > L.cap) return AMSKV_ERR_ARENA_TOO_SMALL;  // cannot happen: cap is the max over steps
  } else {
    cur.off = -1;
    cur.ext_k = K_dev;
    cur.ext_v = V_dev;
  }
  const bool defer = keep_copy && c->fuse != 0;  // the attend call of this step writes the slot
  if (defer) {
    cur.pending = true;
    cur.ext_k = K_dev;
    cur.ext_v = V_dev;
  }
  next.push_back(cur);

  const bool copy_now = keep_copy && !defer;
  if (K_dev && (copy_now || mv.n > 0)) {
    hipError_t e = amskv::launch_append(c->arena + L.k_off, c->arena + L.v_off, copy_now ? K_dev : nullptr,
                                        copy_now ? V_dev : nullptr, bh, row_bytes, L.cap, mv, cur.len,
                                        copy_now ? cur.off : 0, 0, caller_map(c, cur.len, c->kv_tok), c->heads,
                                        (hipStream_t)stream);
    if (e != hipSuccess) return AMSKV_ERR_HIP;
  }
  L.segs.swap(next);
  L.last_evicted.swap(evicted);
  L.last_scale = s;
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

static int density_launch(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, hipStream_t st, SegTable* table,
                          float** totals, float* out_dev);

// The attention of step s; with mass_out_dev also the attention density of the step's queries over the groups of
// keys as they are before the step's own bookkeeping (what amskv_attention_density_enqueue would report just before).
static int attend_step(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, void* O_dev, void* stream,
                       float* mass_out_dev, int32_t* n_seg, int32_t* tok_len) {
  if (bad_layer(c, layer) || s < 0 || s >= c->n_scales || !Q_dev || !O_dev || misaligned(Q_dev) || misaligned(O_dev))
    return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  LayerState& L = c->layer[layer];
  if (s != L.last_scale) return AMSKV_ERR_ORDER;
  // token-budget mode: once the scale's iteration of Algorithm 1 has run it is no longer whole
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET && !L.roll_pending) return AMSKV_ERR_ORDER;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  ExtKV ext;
  const SegTable t = seg_table(L, &ext);
  if (t.ext_start < t.total && !ext.k) return AMSKV_ERR_NO_DEVICE_MEMORY;  // borrowed scale appended without data
  // density: one group per entry of the layer's list; as a by-product of this very launch where the kernel has
  // that form (bf16, more query rows than the coarse-scale kernel takes), else by the stand-alone kernels first
  amskv::GroupEnds groups;
  std::memset(&groups, 0, sizeof(groups));
  bool by_product = false;
  if (mass_out_dev) {
    if (L.segs.size() > (size_t)AMSKV_MAX_SCALES) return AMSKV_ERR_INVALID_ARG;
    by_product = c->dtype == AMSKV_DTYPE_BF16 && amskv::attend_density_fused(c->tokens[s]);
    int32_t v = 0;
    for (const Segment& g : L.segs) {
      v += g.len;
      if (tok_len) tok_len[groups.n] = g.len;
      groups.end[groups.n++] = v;
    }
    *n_seg = groups.n;
    if (!by_product) {
      SegTable pieces;
      float* totals = nullptr;
      if (int rc = density_launch(c, layer, s, Q_dev, (hipStream_t)stream, &pieces, &totals, mass_out_dev)) return rc;
    }
  }
  Segment& newest = L.segs.back();
  if (newest.pending) {  // fused append: this launch also fills the slot
    ext.wb_from = t.ext_start;
    ext.wb_delta = newest.off - t.ext_start;
  }
  // Token modes: whenever the outcome of the step's iteration of Algorithm 1 is known before the step runs, the
  // same launch does its device side.  The scale fits the budget in force next to what is cached: it is written,
  // whole, right behind the cached tokens.  It overflows, no Eq. 3 test is due (the budget cannot grow any more,
  // or there is only one) and one workgroup or wave owns each (b,h): the survivors of Algorithm 2 -- the first
  // c_cds tokens of the list stay where they are, the last budget - c_cds slide down behind them -- are written
  // to their new places as they pass through the kernel, cached rows and rows of the new scale alike (the cached
  // tokens are one run from offset 0, so a token's place in the list is its offset).
  // (Not after the last scale of the schedule: no step follows that would read the result, and left to the next
  // call the iteration is dropped by the reset that ends the image.)
  int on_device = kRollNone;
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET && s + 1 < c->n_scales) {
    int64_t n_old = 0;
    bool one_run = true;
    for (size_t i = 0; i + 1 < L.segs.size(); ++i) {
      one_run = one_run && L.segs[i].off == n_old;
      n_old += L.segs[i].len;
    }
    const int64_t total = n_old + newest.len;
    const int32_t bgt = L.c_bgt;
    const bool cache_it = c->cut_oversize || newest.len <= L.bud.c_max;
    const bool overflow = cache_it && total > bgt;
    const bool wants_test = overflow && bgt == L.bud.c_min && L.bud.c_max > L.bud.c_min;
    const bool one_owner = c->dtype == AMSKV_DTYPE_BF16 && (by_product ? c->tokens[s] <= 128 : amskv::attend_owns_unit(c->head_dim, c->tokens[s]));
    // what the launch writes under budget b: nothing (the scale is larger than the budget and is not cached), the
    // whole scale behind the cached tokens, or Algorithm 2's survivors
    auto plan = [&](int32_t b, int32_t* from, int32_t* delta, int32_t* head_end) {
      *from = amskv::kNoWriteBack;
      *delta = *head_end = 0;
      if (newest.len > b && !c->cut_oversize) return;
      if (total <= b) {
        *from = t.ext_start;
        return;
      }
      *head_end = L.bud.c_cds;
      *from = (int32_t)(total - (b - L.bud.c_cds));
      *delta = *head_end - *from;
    };
    if (cache_it && !overflow) {
      ext.wb_from = t.ext_start;
      ext.wb_delta = 0;
      on_device = kRollAppended;
    } else if (overflow && one_owner && one_run && t.ext_start == n_old) {
      if (!wants_test) {
        plan(bgt, &ext.wb_from, &ext.wb_delta, &ext.wb_head_end);
        on_device = kRollTrimmed;
      } else {
        // the test goes in front of the launch; if it needs the device, the launch is given both outcomes
        int state = kTestFails;
        if (int rc = start_theta_test(c, L, newest, (hipStream_t)stream, &state)) return rc;
        if (state == kTestEnqueued) {
          plan(bgt, &ext.wb_from, &ext.wb_delta, &ext.wb_head_end);
          plan(L.bud.c_max, &ext.alt_from, &ext.alt_delta, &ext.alt_head_end);
          ext.alt_if = theta_flag_dev(c, layer);
          L.test_pending = true;
          on_device = kRollEitherWay;
        } else {
          plan(state == kTestHolds ? L.bud.c_max : bgt, &ext.wb_from, &ext.wb_delta, &ext.wb_head_end);
          on_device = kRollTrimmed;
        }
      }
    }
  }
  const int bh = c->batch * c->heads;
  // the scale read in place, if any, is the newest one
  const CallerIo io{caller_map(c, c->tokens[s], c->q_tok), caller_map(c, c->tokens[s], c->o_tok),
                    caller_map(c, newest.len, c->kv_tok), c->heads};
  hipError_t e;
  if (by_product)
    e = amskv::launch_attend_density_bf16(Q_dev, O_dev, c->arena + L.k_off, c->arena + L.v_off, c->batch, c->heads,
                                          c->tokens[s], c->head_dim, L.cap, t, ext, io, c->softmax_scale, groups,
                                          (float*)(c->arena + c->dens_off), mass_out_dev, (hipStream_t)stream);
  else if (c->dtype == AMSKV_DTYPE_BF16)
    e = amskv::launch_attend_bf16(Q_dev, O_dev, c->arena + L.k_off, c->arena + L.v_off, bh,
                                  c->tokens[s], c->head_dim, L.cap, t, ext, io, c->softmax_scale,
                                  (hipStream_t)stream);
  else
    e = amskv::launch_attend_f32(Q_dev, O_dev, c->arena + L.k_off, c->arena + L.v_off, bh,
                                 c->tokens[s], c->head_dim, L.cap, t, ext, io, c->softmax_scale,
                                 (hipStream_t)stream);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  if (newest.pending) {  // from here on (in stream order) the slot holds the scale
    newest.pending = false;
    newest.ext_k = newest.ext_v = nullptr;
  }
  // what is left of the iteration (anything, unless this launch wrote the whole scale to its place) waits for the next call on the layer
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET) return roll_budget(c, L, (hipStream_t)stream, on_device, true);
  return AMSKV_OK;
}

int32_t amskv_attend(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, void* O_dev, void* stream) try {
  return attend_step(c, layer, s, Q_dev, O_dev, stream, nullptr, nullptr, nullptr);
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_attend_density(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, void* O_dev, float* mass_out_dev,
                             int32_t* n_seg, int32_t* tok_len, void* stream) try {
  if (!mass_out_dev || misaligned(mass_out_dev) || !n_seg) return AMSKV_ERR_INVALID_ARG;
  return attend_step(c, layer, s, Q_dev, O_dev, stream, mass_out_dev, n_seg, tok_len);
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

// Checks shared by the two ways of asking for Eq. 3; on success cur/prev point at the two whole scales.
static int similarity_operands(amskv_cache* c, int32_t layer, int32_t s, const Segment** cur, const Segment** prev) {
  if (bad_layer(c, layer) || s < 1 || s >= c->n_scales) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  LayerState& L = c->layer[layer];
  if (s > L.last_scale) return AMSKV_ERR_ORDER;
  *cur = *prev = nullptr;
  for (const Segment& g : L.segs) {
    if (whole_scale(c, g, s)) *cur = &g;
    if (whole_scale(c, g, s - 1)) *prev = &g;
  }
  if (!*cur || !*prev) return AMSKV_ERR_EVICTED;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  if ((((*cur)->off < 0 || (*cur)->pending) && !(*cur)->ext_k) || (((*prev)->off < 0 || (*prev)->pending) && !(*prev)->ext_k))
    return AMSKV_ERR_NO_DEVICE_MEMORY;
  return AMSKV_OK;
}

static void similarity_outputs(const amskv_cache* c, int s, bool has_v, const float* sums, float* cosK, float* cosV,
                               float* sums_out) {
  const double n_tok = (double)c->batch * c->tokens[s];
  for (int h = 0; h < c->heads; ++h) {
    if (cosK) cosK[h] = (float)(sums[h * 4 + 0] / n_tok);
    if (sums_out) {
      sums_out[h * 3 + 0] = sums[h * 4 + 1];
      sums_out[h * 3 + 1] = sums[h * 4 + 2];
      sums_out[h * 3 + 2] = sums[h * 4 + 3];
    }
    if (cosV) cosV[h] = has_v ? (float)(sums[(c->heads + h) * 4 + 0] / n_tok) : NAN;
  }
}

int32_t amskv_interscale_similarity(amskv_cache* c, int32_t layer, int32_t s, float* cosK_host,
                                    float* cosV_host, float* sums_host, void* stream) try {
  if (!cosK_host) return AMSKV_ERR_INVALID_ARG;
  const Segment *cur, *prev;
  int rc = similarity_operands(c, layer, s, &cur, &prev);
  if (rc) return rc;
  std::vector<float> host;
  rc = similarity_sums(c, c->layer[layer], layer, *cur, *prev, s, cosV_host != nullptr, &host, (hipStream_t)stream);
  if (rc) return rc;
  similarity_outputs(c, s, cosV_host != nullptr, host.data(), cosK_host, cosV_host, sums_host);
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_interscale_similarity_enqueue(amskv_cache* c, int32_t layer, int32_t s, int32_t want_v, void* stream) try {
  const Segment *cur, *prev;
  int rc = similarity_operands(c, layer, s, &cur, &prev);
  if (rc) return rc;
  return similarity_launch(c, c->layer[layer], layer, *cur, *prev, s, want_v != 0, (hipStream_t)stream);
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_interscale_similarity_enqueue_static(amskv_cache* c, int32_t layer, int32_t s, int32_t want_v,
                                                   float* sums_out_dev, void* stream) try {
  if (!sums_out_dev || misaligned(sums_out_dev)) return AMSKV_ERR_INVALID_ARG;
  const Segment *cur, *prev;
  int rc = similarity_operands(c, layer, s, &cur, &prev);
  if (rc) return rc;
  if ((int64_t)c->batch * c->heads > AMSKV_STATIC_MAX_UNITS) return AMSKV_ERR_STATIC_LIMIT;
  const LayerState& L = c->layer[layer];
  hipError_t e = amskv::launch_similarity_static(scale_ref(c, L, *cur, want_v != 0), scale_ref(c, L, *prev, want_v != 0),
                                                 c->batch, c->heads, c->head_dim, c->dtype, c->side_h[s], c->side_w[s],
                                                 c->side_h[s - 1], c->side_w[s - 1], sums_out_dev, (hipStream_t)stream);
  return e == hipSuccess ? AMSKV_OK : AMSKV_ERR_HIP;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_interscale_similarity_collect(amskv_cache* c, float* cosK_host, float* cosV_host, float* sums_host,
                                            void* stream) try {
  if (!c || !cosK_host) return AMSKV_ERR_INVALID_ARG;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  const size_t per_layer = 2 * (size_t)c->heads * 4;
  std::vector<float> host(per_layer * c->layers);
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(host.data(), similarity_slot(c, 0), host.size() * sizeof(float), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  for (int l = 0; l < c->layers; ++l) {
    const LayerState& L = c->layer[l];
    float* ck = cosK_host + (size_t)l * c->heads;
    float* cv = cosV_host ? cosV_host + (size_t)l * c->heads : nullptr;
    float* sm = sums_host ? sums_host + (size_t)l * c->heads * 3 : nullptr;
    if (L.sim_scale < 1) {  // nothing enqueued on this layer since create / reset
      for (int h = 0; h < c->heads; ++h) {
        ck[h] = NAN;
        if (cv) cv[h] = NAN;
        if (sm) sm[h * 3] = sm[h * 3 + 1] = sm[h * 3 + 2] = NAN;
      }
      continue;
    }
    similarity_outputs(c, L.sim_scale, L.sim_has_v, host.data() + per_layer * l, ck, cv, sm);
  }
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

// Checks and launch shared by the forms of the density call; the per-head masses end up at out_dev, or, when that
// is null, inside the arena's workspace; *totals is where, and *table describes the groups.
static int density_launch(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, hipStream_t st, SegTable* table,
                          float** totals, float* out_dev) {
  if (bad_layer(c, layer) || s < 0 || s >= c->n_scales || !Q_dev || misaligned(Q_dev)) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  LayerState& L = c->layer[layer];
  if (s != L.last_scale) return AMSKV_ERR_ORDER;
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET && !L.roll_pending) return AMSKV_ERR_ORDER;
  if (L.segs.size() > (size_t)AMSKV_MAX_SCALES) return AMSKV_ERR_INVALID_ARG;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  ExtKV ext;
  const SegTable t = seg_table(L, &ext, false);  // one entry per group of keys, nothing merged
  if (t.ext_start < t.total && !ext.k) return AMSKV_ERR_NO_DEVICE_MEMORY;
  const int64_t n_qblk = (c->tokens[s] + 31) / 32;
  if ((int64_t)c->batch * c->heads * n_qblk > INT32_MAX) return AMSKV_ERR_INVALID_ARG;
  float* partial = (float*)(c->arena + c->dens_off);
  *totals = out_dev ? out_dev : partial + (uint64_t)c->batch * c->heads * n_qblk * AMSKV_MAX_SCALES;
  const CallerIo io{caller_map(c, c->tokens[s], c->q_tok), RowMap{0, 0, 0}, caller_map(c, L.segs.back().len, c->kv_tok),
                    c->heads};
  hipError_t e = amskv::launch_density(Q_dev, c->arena + L.k_off, c->batch, c->heads, c->tokens[s], c->head_dim, c->dtype,
                                       L.cap, t, ext, io, c->softmax_scale, partial, *totals, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  *table = t;
  return AMSKV_OK;
}

int32_t amskv_attention_density(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, float* density_host,
                                float* mass_host, int32_t* n_seg, void* stream) try {
  if (!density_host && !mass_host) return AMSKV_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  SegTable t;
  float* totals = nullptr;
  int rc = density_launch(c, layer, s, Q_dev, st, &t, &totals, nullptr);
  if (rc) return rc;
  std::vector<float> host((size_t)c->heads * AMSKV_MAX_SCALES);
  hipError_t e = hipMemcpyAsync(host.data(), totals, host.size() * sizeof(float), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  for (int h = 0; h < c->heads; ++h)
    for (int p = 0; p < t.n; ++p) {
      const float m = host[(size_t)h * AMSKV_MAX_SCALES + p];
      if (mass_host) mass_host[h * AMSKV_MAX_SCALES + p] = m;
      if (density_host) density_host[h * AMSKV_MAX_SCALES + p] = m / (float)t.len[p];
    }
  if (n_seg) *n_seg = t.n;
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_attention_density_enqueue(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, float* mass_out_dev,
                                        int32_t* n_seg, int32_t* tok_len, void* stream) try {
  if (!mass_out_dev || misaligned(mass_out_dev) || !n_seg) return AMSKV_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  SegTable t;
  float* totals = nullptr;
  int rc = density_launch(c, layer, s, Q_dev, st, &t, &totals, mass_out_dev);
  if (rc) return rc;
  *n_seg = t.n;
  if (tok_len)
    for (int p = 0; p < t.n; ++p) tok_len[p] = t.len[p];
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_layout(const amskv_cache* c, int32_t layer, int32_t* n_seg, int32_t* scale_id,
                           int64_t* tok_offset, int32_t* tok_len) try {
  if (bad_layer(c, layer) || !n_seg) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  *n_seg = (int32_t)L.segs.size();
  for (size_t i = 0; i < L.segs.size(); ++i) {
    if (scale_id) scale_id[i] = L.segs[i].scale;
    if (tok_offset) tok_offset[i] = L.segs[i].off;
    if (tok_len) tok_len[i] = L.segs[i].len;
  }
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_segments(const amskv_cache* c, int32_t layer, int32_t* n_seg, int32_t* scale_id,
                             int32_t* first_token, int64_t* tok_offset, int32_t* tok_len) try {
  if (bad_layer(c, layer) || !n_seg) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  *n_seg = (int32_t)L.segs.size();
  for (size_t i = 0; i < L.segs.size(); ++i) {
    if (scale_id) scale_id[i] = L.segs[i].scale;
    if (first_token) first_token[i] = L.segs[i].first;
    if (tok_offset) tok_offset[i] = L.segs[i].off;
    if (tok_len) tok_len[i] = L.segs[i].len;
  }
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int64_t amskv_cache_budget_tokens(const amskv_cache* c, int32_t layer) {
  if (bad_layer(c, layer)) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  return c->mode == AMSKV_MODE_TOKEN_BUDGET ? (int64_t)L.c_bgt : L.cap;
}

int32_t amskv_cache_settle(amskv_cache* c, int32_t layer, void* stream) try {
  if (bad_layer(c, layer)) return AMSKV_ERR_INVALID_ARG;
  LayerState& L = c->layer[layer];
  if (c->mode == AMSKV_MODE_TOKEN_BUDGET) return roll_budget(c, L, (hipStream_t)stream);
  return flush_pending(c, L, (hipStream_t)stream);
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_last_evicted(const amskv_cache* c, int32_t layer, int32_t* n_evicted,
                                 int32_t* scale_id) try {
  if (bad_layer(c, layer) || !n_evicted) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  *n_evicted = (int32_t)L.last_evicted.size();
  if (scale_id)
    for (size_t i = 0; i < L.last_evicted.size(); ++i) scale_id[i] = L.last_evicted[i];
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int64_t amskv_cache_bytes_held(const amskv_cache* c, int32_t layer, int32_t include_current) {
  if (bad_layer(c, layer)) return AMSKV_ERR_INVALID_ARG;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  int64_t tok = 0;
  for (const Segment& g : L.segs)
    if (include_current || g.scale != L.last_scale) tok += g.len;
  return 2 * (int64_t)c->elem_bytes * c->batch * c->heads * c->head_dim * tok;
}

int64_t amskv_cache_capacity_tokens(const amskv_cache* c, int32_t layer) {
  if (bad_layer(c, layer)) return AMSKV_ERR_INVALID_ARG;
  return c->layer[layer].cap;
}

int32_t amskv_cache_export(const amskv_cache* c, int32_t layer, void* K_out_dev, void* V_out_dev,
                           void* stream) try {
  if (bad_layer(c, layer) || (!K_out_dev && !V_out_dev)) return AMSKV_ERR_INVALID_ARG;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  if (int rc = finish_iteration(c, layer)) return rc;
  const LayerState& L = c->layer[layer];
  if (L.segs.empty()) return AMSKV_OK;
  ExtKV ext;
  const SegTable t = seg_table(L, &ext);
  if (t.ext_start < t.total && !ext.k) return AMSKV_ERR_NO_DEVICE_MEMORY;
  hipError_t e = amskv::launch_export(c->arena + L.k_off, c->arena + L.v_off, K_out_dev, V_out_dev,
                                      c->batch * c->heads, c->head_dim * c->elem_bytes, L.cap, t, ext,
                                      caller_map(c, L.segs.back().len, c->kv_tok), c->heads, (hipStream_t)stream);
  return e == hipSuccess ? AMSKV_OK : AMSKV_ERR_HIP;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_set_io_layout(amskv_cache* c, int32_t io_layout, int64_t q_token_stride, int64_t kv_token_stride,
                                  int64_t o_token_stride) try {
  if (!c || (io_layout != AMSKV_IO_HEAD_MAJOR && io_layout != AMSKV_IO_TOKEN_MAJOR)) return AMSKV_ERR_INVALID_ARG;
  for (const LayerState& L : c->layer)
    if (L.last_scale >= 0) return AMSKV_ERR_ORDER;  // recorded K/V pointers would change meaning
  if (io_layout == AMSKV_IO_TOKEN_MAJOR) {
    const int64_t width = (int64_t)c->heads * c->head_dim, per16 = 16 / c->elem_bytes;
    for (int64_t st : {q_token_stride, kv_token_stride, o_token_stride})
      if (st < width || st % per16 != 0 || st > ((int64_t)1 << 40)) return AMSKV_ERR_INVALID_ARG;
    c->q_tok = q_token_stride;
    c->kv_tok = kv_token_stride;
    c->o_tok = o_token_stride;
  } else {
    c->q_tok = c->kv_tok = c->o_tok = 0;
  }
  c->io_layout = io_layout;
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

int32_t amskv_cache_reset(amskv_cache* c) try {
  if (!c) return AMSKV_ERR_INVALID_ARG;
  for (LayerState& L : c->layer) {
    L.segs.clear();
    L.last_evicted.clear();
    L.last_scale = -1;
    L.c_bgt = L.bud.c_min;
    L.roll_pending = false;
    L.deferred = L.test_pending = L.device_done = false;  // an enqueued test still runs; its result is not read
    L.sim_scale = -1;
  }
  return AMSKV_OK;
} catch (const std::bad_alloc&) {
  return AMSKV_ERR_NO_HOST_MEMORY;  // nothing of the call may have taken effect on the host state that matters: callers destroy the cache
}

void amskv_cache_destroy(amskv_cache* c) {
  if (!c) return;
  for (LayerState& L : c->layer)
    if (L.test_done) {
      (void)hipEventSynchronize(L.test_done);  // a kernel that writes into theta_host may still be in flight
      (void)hipEventDestroy(L.test_done);
    }
  if (c->theta_host) (void)hipHostFree(c->theta_host);
  delete c;
}

}  // extern "C"
