// Host layer of libamskv: schedule, per-layer policy -> kept set, arena layout, segment
// tables, status codes, and the C ABI declared in amskv.h.  All policy decisions are made
// here on the host; the kernels only see token offsets.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "amskv_internal.hpp"

namespace {

using amskv::ExtKV;
using amskv::MoveList;
using amskv::ScaleRef;
using amskv::SegTable;

struct Segment {
  int32_t scale;
  int32_t off;  // token offset inside the layer's [cap] axis; -1: borrowed (read in place)
  int32_t len;
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
};

}  // namespace

struct amskv_cache {
  int32_t layers, heads, head_dim, batch, dtype, n_scales, layout, borrow, fuse;
  int32_t side_h[AMSKV_MAX_SCALES], side_w[AMSKV_MAX_SCALES], tokens[AMSKV_MAX_SCALES];
  float softmax_scale;
  int32_t elem_bytes;
  char* arena = nullptr;
  uint64_t arena_bytes = 0;
  uint64_t ws_off = 0;  // similarity workspace
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
  if (po->n_layers != layers || !po->layer) return AMSKV_ERR_INVALID_ARG;
  if (po->layout != AMSKV_LAYOUT_COMPACT && po->layout != AMSKV_LAYOUT_PLANNED)
    return AMSKV_ERR_INVALID_ARG;
  if (po->borrow_unretained != 0 && po->borrow_unretained != 1) return AMSKV_ERR_INVALID_ARG;
  if (po->fuse_append != 0 && po->fuse_append != 1) return AMSKV_ERR_INVALID_ARG;
  if (!(po->softmax_scale >= 0.f) || !std::isfinite(po->softmax_scale)) return AMSKV_ERR_INVALID_ARG;
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
// scales with overlapping lifetimes never overlap in memory (largest scale first, lowest free
// offset), so eviction needs no data movement at all.  Returns the capacity reached.
int64_t plan_slots(const amskv_layer_policy& p, const int32_t* tokens, int n_scales, bool borrow,
                   int32_t* off_out) {
  std::vector<int> order;
  for (int i = 0; i < n_scales; ++i) {
    off_out[i] = -1;
    if (stored(p, i, n_scales, borrow)) order.push_back(i);
  }
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return tokens[a] > tokens[b]; });
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

struct Plan {
  std::vector<int64_t> cap;
  std::vector<uint64_t> k_off, v_off;
  std::vector<std::vector<int32_t>> slot;
  uint64_t ws_off = 0, total = 0;
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
    if (po->layout == AMSKV_LAYOUT_PLANNED)
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
  // similarity workspace: per (tensor, b, h) four partial sums, then per (tensor, h) four totals
  at = align_up(at + (2 * bh * 4 + 2 * (uint64_t)heads * 4) * sizeof(float));
  pl->total = at;
}

inline bool bad_layer(const amskv_cache* c, int32_t layer) {
  return !c || layer < 0 || layer >= c->layers;
}

// Segment table for the kernels; a borrowed segment (always the newest scale, hence last)
// becomes the external tail of the virtual concatenation.
SegTable seg_table(const LayerState& L, ExtKV* ext) {
  SegTable t;
  std::memset(&t, 0, sizeof(t));
  ext->k = ext->v = nullptr;
  ext->wb_off = -1;
  t.n = (int32_t)L.segs.size();
  int32_t v = 0;
  int32_t ext_start = -1;
  for (int i = 0; i < t.n; ++i) {
    t.virt_start[i] = v;
    t.phys_off[i] = L.segs[i].off < 0 ? 0 : L.segs[i].off;
    t.len[i] = L.segs[i].len;
    if (L.segs[i].off < 0 || L.segs[i].pending) {
      ext_start = v;
      ext->k = L.segs[i].ext_k;
      ext->v = L.segs[i].ext_v;
    }
    v += L.segs[i].len;
  }
  t.total = v;
  t.ext_start = ext_start < 0 ? v : ext_start;
  return t;
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
    default: return "unknown status";
  }
}

int32_t amskv_cache_required_bytes(int32_t layers, int32_t heads, int32_t head_dim,
                                   const amskv_schedule* sc, const amskv_policy* po,
                                   uint64_t* bytes_out) {
  if (!bytes_out) return AMSKV_ERR_INVALID_ARG;
  int rc = validate(layers, heads, head_dim, sc, po);
  if (rc) return rc;
  Plan pl;
  build_plan(layers, heads, head_dim, sc, po, &pl);
  *bytes_out = pl.total;
  return AMSKV_OK;
}

int32_t amskv_cache_create(int32_t layers, int32_t heads, int32_t head_dim,
                           const amskv_schedule* sc, const amskv_policy* po, void* arena_dev,
                           uint64_t arena_bytes, amskv_cache** out) {
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
  if (!c) return AMSKV_ERR_INVALID_ARG;
  c->layers = layers;
  c->heads = heads;
  c->head_dim = head_dim;
  c->batch = sc->batch;
  c->dtype = sc->dtype;
  c->n_scales = sc->n_scales;
  c->layout = po->layout;
  c->borrow = po->borrow_unretained;
  c->fuse = po->fuse_append;
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
  c->layer.resize(layers);
  for (int l = 0; l < layers; ++l) {
    LayerState& L = c->layer[l];
    L.pol = po->layer[l];
    L.cap = pl.cap[l];
    L.k_off = pl.k_off[l];
    L.v_off = pl.v_off[l];
    for (int i = 0; i < AMSKV_MAX_SCALES; ++i) L.planned_off[i] = pl.slot[l][i];
  }
  *out = c;
  return AMSKV_OK;
}

int32_t amskv_append_scale(amskv_cache* c, int32_t layer, int32_t s, const void* K_dev,
                           const void* V_dev, void* stream) {
  if (bad_layer(c, layer) || s < 0 || s >= c->n_scales) return AMSKV_ERR_INVALID_ARG;
  if ((K_dev == nullptr) != (V_dev == nullptr)) return AMSKV_ERR_INVALID_ARG;
  LayerState& L = c->layer[layer];
  if (s != L.last_scale + 1) return AMSKV_ERR_ORDER;
  if (K_dev && !c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;

  const int bh = c->batch * c->heads;
  const int row_bytes = c->head_dim * c->elem_bytes;
  // fuse_append: a scale whose attend never came still lives only in the caller's buffers; copy it now
  for (Segment& g : L.segs) {
    if (!g.pending) continue;
    if (g.ext_k) {
      MoveList none;
      std::memset(&none, 0, sizeof(none));
      hipError_t e = amskv::launch_append(c->arena + L.k_off, c->arena + L.v_off, g.ext_k, g.ext_v, bh, row_bytes,
                                          L.cap, none, g.len, g.off, (hipStream_t)stream);
      if (e != hipSuccess) return AMSKV_ERR_HIP;
    }
    g.pending = false;
    g.ext_k = g.ext_v = nullptr;
  }

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
                                        copy_now ? cur.off : 0, (hipStream_t)stream);
    if (e != hipSuccess) return AMSKV_ERR_HIP;
  }
  L.segs.swap(next);
  L.last_evicted.swap(evicted);
  L.last_scale = s;
  return AMSKV_OK;
}

int32_t amskv_attend(amskv_cache* c, int32_t layer, int32_t s, const void* Q_dev, void* O_dev,
                     void* stream) {
  if (bad_layer(c, layer) || s < 0 || s >= c->n_scales || !Q_dev || !O_dev)
    return AMSKV_ERR_INVALID_ARG;
  LayerState& L = c->layer[layer];
  if (s != L.last_scale) return AMSKV_ERR_ORDER;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  ExtKV ext;
  const SegTable t = seg_table(L, &ext);
  if (t.ext_start < t.total && !ext.k) return AMSKV_ERR_NO_DEVICE_MEMORY;  // borrowed scale appended without data
  Segment& newest = L.segs.back();
  if (newest.pending) ext.wb_off = newest.off;  // fused append: this launch also fills the slot
  const int bh = c->batch * c->heads;
  hipError_t e;
  if (c->dtype == AMSKV_DTYPE_BF16)
    e = amskv::launch_attend_bf16(Q_dev, O_dev, c->arena + L.k_off, c->arena + L.v_off, bh,
                                  c->tokens[s], c->head_dim, L.cap, t, ext, c->softmax_scale,
                                  (hipStream_t)stream);
  else
    e = amskv::launch_attend_f32(Q_dev, O_dev, c->arena + L.k_off, c->arena + L.v_off, bh,
                                 c->tokens[s], c->head_dim, L.cap, t, ext, c->softmax_scale,
                                 (hipStream_t)stream);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  if (newest.pending) {  // from here on (in stream order) the slot holds the scale
    newest.pending = false;
    newest.ext_k = newest.ext_v = nullptr;
  }
  return AMSKV_OK;
}

int32_t amskv_interscale_similarity(amskv_cache* c, int32_t layer, int32_t s, float* cosK_host,
                                    float* cosV_host, float* sums_host, void* stream) {
  if (bad_layer(c, layer) || s < 1 || s >= c->n_scales || !cosK_host) return AMSKV_ERR_INVALID_ARG;
  LayerState& L = c->layer[layer];
  if (s > L.last_scale) return AMSKV_ERR_ORDER;
  const Segment* cur = nullptr;
  const Segment* prev = nullptr;
  for (const Segment& g : L.segs) {
    if (g.scale == s) cur = &g;
    if (g.scale == s - 1) prev = &g;
  }
  if (!cur || !prev) return AMSKV_ERR_EVICTED;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  if (((cur->off < 0 || cur->pending) && !cur->ext_k) || ((prev->off < 0 || prev->pending) && !prev->ext_k))
    return AMSKV_ERR_NO_DEVICE_MEMORY;
  const uint64_t bh = (uint64_t)c->batch * c->heads;
  float* partial = (float*)(c->arena + c->ws_off);
  float* totals = partial + 2 * bh * 4;
  hipStream_t st = (hipStream_t)stream;
  auto ref = [&](const Segment* g) {
    ScaleRef r;
    if (g->off < 0 || g->pending) {
      r.k = g->ext_k;
      r.v = cosV_host ? g->ext_v : nullptr;
      r.stride_tokens = g->len;
      r.off_tokens = 0;
    } else {
      r.k = c->arena + L.k_off;
      r.v = cosV_host ? c->arena + L.v_off : nullptr;
      r.stride_tokens = L.cap;
      r.off_tokens = g->off;
    }
    return r;
  };
  hipError_t e = amskv::launch_similarity(ref(cur), ref(prev), c->batch, c->heads, c->head_dim, c->dtype,
                                          c->side_h[s], c->side_w[s], c->side_h[s - 1], c->side_w[s - 1],
                                          partial, totals, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  std::vector<float> host(2 * (size_t)c->heads * 4);
  const size_t n_t = cosV_host ? 2 : 1;
  e = hipMemcpyAsync(host.data(), totals, n_t * c->heads * 4 * sizeof(float), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return AMSKV_ERR_HIP;
  const double n_tok = (double)c->batch * c->tokens[s];
  for (int h = 0; h < c->heads; ++h) {
    cosK_host[h] = (float)(host[h * 4 + 0] / n_tok);
    if (sums_host) {
      sums_host[h * 3 + 0] = host[h * 4 + 1];
      sums_host[h * 3 + 1] = host[h * 4 + 2];
      sums_host[h * 3 + 2] = host[h * 4 + 3];
    }
    if (cosV_host) cosV_host[h] = (float)(host[(c->heads + h) * 4 + 0] / n_tok);
  }
  return AMSKV_OK;
}

int32_t amskv_cache_layout(const amskv_cache* c, int32_t layer, int32_t* n_seg, int32_t* scale_id,
                           int64_t* tok_offset, int32_t* tok_len) {
  if (bad_layer(c, layer) || !n_seg) return AMSKV_ERR_INVALID_ARG;
  const LayerState& L = c->layer[layer];
  *n_seg = (int32_t)L.segs.size();
  for (size_t i = 0; i < L.segs.size(); ++i) {
    if (scale_id) scale_id[i] = L.segs[i].scale;
    if (tok_offset) tok_offset[i] = L.segs[i].off;
    if (tok_len) tok_len[i] = L.segs[i].len;
  }
  return AMSKV_OK;
}

int32_t amskv_cache_last_evicted(const amskv_cache* c, int32_t layer, int32_t* n_evicted,
                                 int32_t* scale_id) {
  if (bad_layer(c, layer) || !n_evicted) return AMSKV_ERR_INVALID_ARG;
  const LayerState& L = c->layer[layer];
  *n_evicted = (int32_t)L.last_evicted.size();
  if (scale_id)
    for (size_t i = 0; i < L.last_evicted.size(); ++i) scale_id[i] = L.last_evicted[i];
  return AMSKV_OK;
}

int64_t amskv_cache_bytes_held(const amskv_cache* c, int32_t layer, int32_t include_current) {
  if (bad_layer(c, layer)) return AMSKV_ERR_INVALID_ARG;
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
                           void* stream) {
  if (bad_layer(c, layer) || (!K_out_dev && !V_out_dev)) return AMSKV_ERR_INVALID_ARG;
  if (!c->arena) return AMSKV_ERR_NO_DEVICE_MEMORY;
  const LayerState& L = c->layer[layer];
  if (L.segs.empty()) return AMSKV_OK;
  ExtKV ext;
  const SegTable t = seg_table(L, &ext);
  if (t.ext_start < t.total && !ext.k) return AMSKV_ERR_NO_DEVICE_MEMORY;
  hipError_t e = amskv::launch_export(c->arena + L.k_off, c->arena + L.v_off, K_out_dev, V_out_dev,
                                      c->batch * c->heads, c->head_dim * c->elem_bytes, L.cap, t, ext,
                                      (hipStream_t)stream);
  return e == hipSuccess ? AMSKV_OK : AMSKV_ERR_HIP;
}

int32_t amskv_cache_reset(amskv_cache* c) {
  if (!c) return AMSKV_ERR_INVALID_ARG;
  for (LayerState& L : c->layer) {
    L.segs.clear();
    L.last_evicted.clear();
    L.last_scale = -1;
  }
  return AMSKV_OK;
}

void amskv_cache_destroy(amskv_cache* c) { delete c; }

}  // extern "C"
