/*
 * amskv.h -- C ABI of the AMS-KV hot path for AMD MI355X (gfx950).
 *
 * AMS-KV (arxiv 2511.16047) is a per-layer KV-cache policy for next-scale-prediction
 * visual autoregressive transformers: an image is generated as S scales of h_s x w_s
 * tokens (Section 3.1, Eq. 1-2); the tokens of scale s attend to every cached earlier
 * scale and, bidirectionally, to their own scale.  Each layer keeps the first few
 * "condensed" scales for good, a rolling window of "local" scales just before the
 * current one, and drops the "intermediate" ones (Section 4.1, Section 4.3, Algorithm 2);
 * layers whose adjacent-scale keys are dissimilar (Eq. 3) are "cache-demanding" and keep
 * more (Section 4.2).
 *
 * This library owns only host-side metadata.  All device memory -- the inputs, the
 * outputs and the cache arena -- is allocated by the caller and passed as plain device
 * pointers.  Every call that touches device memory enqueues its kernels on the
 * hipStream_t passed as `stream` (NULL = the null stream) and returns without waiting,
 * except where stated.  No call allocates or frees device memory.
 *
 * Tensor layouts (all row-major, contiguous):
 *   Q, K, V, O of scale s : [B][H][T_s][D],  T_s = side_h[s]*side_w[s], tokens of a scale
 *                           in row-major grid order (or token-major, amskv_cache_set_io_layout)
 *   cache of layer l      : K[B][H][cap_l][D] followed by V[B][H][cap_l][D] inside the
 *                           arena; the kept scales sit back to back in ascending scale
 *                           order (AMSKV_LAYOUT_COMPACT) or at offsets fixed at create
 *                           time (AMSKV_LAYOUT_PLANNED); amskv_cache_layout reports them
 * Element type: float (dtype 0) or bfloat16 (dtype 1), the same for every tensor.
 *
 * Every function returns an amskv_status (0 = ok, negative = error) unless stated.
 * On error nothing has been enqueued and the cache state is unchanged; the one exception is
 * AMSKV_ERR_HIP (a failed launch or copy may follow work already enqueued by the same call).
 */
#ifndef AMSKV_H
#define AMSKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AMSKV_OK = 0,
  AMSKV_ERR_INVALID_ARG = -1,     /* null pointer, bad size, unsupported head_dim/dtype      */
  AMSKV_ERR_ORDER = -2,           /* scales not appended in order / attend on a stale scale  */
  AMSKV_ERR_EVICTED = -3,         /* the call needs a scale that is not resident             */
  AMSKV_ERR_ARENA_TOO_SMALL = -4, /* arena_bytes < amskv_cache_required_bytes                 */
  AMSKV_ERR_HIP = -5,             /* a HIP runtime call failed (launch, copy, sync)          */
  AMSKV_ERR_NO_DEVICE_MEMORY = -6,/* device work asked of a plan-only cache (arena == NULL)  */
  AMSKV_ERR_STATIC_LIMIT = -7,    /* batch * heads beyond what the static workspace holds    */
  AMSKV_ERR_NO_HOST_MEMORY = -8   /* a host allocation failed; destroy the cache             */
} amskv_status;

enum { AMSKV_DTYPE_F32 = 0, AMSKV_DTYPE_BF16 = 1 };
enum { AMSKV_LAYOUT_COMPACT = 0, AMSKV_LAYOUT_PLANNED = 1 };
enum { AMSKV_MODE_SCALE_WINDOW = 0, AMSKV_MODE_TOKEN_BUDGET = 1, AMSKV_MODE_TOKEN_WINDOW = 2 };
enum { AMSKV_IO_HEAD_MAJOR = 0, AMSKV_IO_TOKEN_MAJOR = 1 };
enum { AMSKV_MAX_SCALES = 16 };
enum { AMSKV_STATIC_MAX_UNITS = 16384 }; /* batch * heads limit of amskv_interscale_similarity_enqueue_static */

typedef struct amskv_cache amskv_cache; /* opaque, host memory, owned by the library */

/* The scale schedule (Section 3.1/3.2): n_scales grids of side_h[s] x side_w[s] tokens,
 * generated in this order.  `batch` is the literal batch B (a caller that doubles the
 * batch for classifier-free guidance passes the doubled value). */
typedef struct {
  int32_t n_scales;       /* 1 .. AMSKV_MAX_SCALES                       */
  const int32_t* side_h;  /* host, [n_scales], each >= 1                  */
  const int32_t* side_w;  /* host, [n_scales], each >= 1                  */
  int32_t batch;          /* B >= 1                                       */
  int32_t dtype;          /* AMSKV_DTYPE_F32 or AMSKV_DTYPE_BF16          */
} amskv_schedule;

/* Per-layer policy in scale units (Section 4.3; Algorithm 2 with budgets counted in whole
 * scales): after scale s is appended the layer holds scales {0..n_condensed-1}, the
 * `window` scales before s, and s, clipped to [0, s].  keep_all != 0 keeps every scale
 * (a cache-demanding layer with an unlimited budget, and the vanilla baseline). */
typedef struct {
  int32_t n_condensed;    /* >= 0 */
  int32_t window;         /* >= 0 */
  int32_t keep_all;       /* 0 / 1 */
} amskv_layer_policy;

/* Per-layer budgets in tokens for AMSKV_MODE_TOKEN_BUDGET: Algorithm 1 and Algorithm 2 taken
 * literally (Section 4.3).  The layer starts with the budget c_min.  At every iteration of
 * Algorithm 1 at which the cached tokens plus the new scale exceed the budget while the budget
 * still is c_min, the layer is tested for being cache-demanding (Eq. 3 score below theta); the
 * first time the test holds the budget becomes c_max for good, and a layer whose test keeps
 * failing is tested again at each later overflowing step (three times on a ten-scale schedule
 * with c_min below the sixth scale's running total).  A scale larger than c_max, or larger than
 * the budget in force, is never cached.  Otherwise the cache keeps its first c_cds tokens and
 * the most recent (budget - c_cds) tokens, so a scale may stay in part.
 * The score compared with theta is the mean over heads of the mean per-token cosine between
 * the keys of the new scale and the bilinearly upsampled keys of the scale before it (the
 * cosine form of Eq. 3 that amskv_interscale_similarity returns as cosK).  It can be computed
 * only while that earlier scale is cached whole; when it is not, the test counts as failed and
 * the budget stays.  theta > 1 always expands and theta < -1 never does, both without device
 * work (the cosine lies in [-1, 1]). */
typedef struct {
  int32_t c_min;          /* >= c_cds           */
  int32_t c_max;          /* >= c_min, >= 1     */
  int32_t c_cds;          /* >= 0               */
  float theta;
} amskv_layer_budget;

typedef struct {
  int32_t n_layers;                 /* must equal `layers` of the create call            */
  const amskv_layer_policy* layer;  /* host, [n_layers]; unused (may be NULL) in token-budget mode */
  float softmax_scale;              /* 0 => 1/sqrt(head_dim)                              */
  int32_t layout;                   /* AMSKV_LAYOUT_COMPACT or AMSKV_LAYOUT_PLANNED       */
  int32_t borrow_unretained;        /* 0 / 1, see below                                   */
  int32_t fuse_append;              /* 0 / 1, see below                                   */
  int32_t mode;                     /* AMSKV_MODE_SCALE_WINDOW (0), _TOKEN_BUDGET or _TOKEN_WINDOW */
  const amskv_layer_budget* budget; /* host, [n_layers]; token-budget and token-window modes */
} amskv_policy;

/* borrow_unretained.  Algorithm 1 stores a scale only if a later step will read it (a scale
 * larger than the budget is skipped, so the final scale is never cached); the attention of the
 * current step still uses that scale's own K/V.  With borrow_unretained != 0 the library does
 * the same: when scale s is appended and the policy does not keep it at step s+1 (always true
 * for the last scale of the schedule), nothing is copied -- the cache records K_dev/V_dev, and
 * amskv_attend, amskv_interscale_similarity and amskv_cache_export read the scale in place.
 * The caller must then keep K_dev/V_dev valid and unchanged until the next append or reset on
 * that layer (or the destroy).  Such a scale needs no arena space (capacities shrink
 * accordingly) and amskv_cache_layout reports it with tok_offset = -1.  With 0 (default) every
 * appended scale is copied and K_dev/V_dev may be reused as soon as the append has run.
 *
 * fuse_append.  The attention of step s streams K_s and V_s anyway, so with fuse_append != 0
 * amskv_append_scale does not copy a retained scale either: it reserves the scale's slot, and
 * the amskv_attend call of that step reads the scale from K_dev/V_dev and writes it into the
 * slot as it goes (one read of K_s/V_s instead of two, and no copy kernel).  If the next call
 * on the layer is another append instead, that append performs the copy first.  Same promise
 * as above: K_dev/V_dev stay valid and unchanged until the next append or reset on the layer;
 * until the attend call they are the only copy, and similarity/export read them in place.
 * Device work of one layer must be enqueued on one stream (or be ordered by the caller).
 *
 * Stream capture.  In scale-window mode amskv_append_scale, amskv_attend, amskv_attend_density,
 * amskv_attention_density_enqueue, amskv_interscale_similarity_enqueue and
 * amskv_interscale_similarity_enqueue_static enqueue kernels
 * only -- no memory copies, memsets, events or waits -- so a caller whose Q, K, V and O live in
 * fixed buffers may issue a whole image's calls (amskv_cache_reset first) on a stream under HIP graph
 * capture and replay the graph per image: the host side of the calls (kept sets, slots, kernel
 * arguments) runs once, at capture, and is the same for every image.  Calls that return results to
 * the host (_collect, the waiting forms, amskv_cache_export to the host's eyes) and the token modes,
 * whose host decisions depend on device results (Eq. 3), are not capturable.
 *
 * mode = AMSKV_MODE_TOKEN_BUDGET.  The cache of a layer is a list of tokens, oldest first, kept
 * back to back from offset 0 of the layer's regions (layout must be AMSKV_LAYOUT_COMPACT,
 * borrow_unretained and fuse_append must be 0; the capacity of a layer is c_max tokens).
 * Step s runs in this order: amskv_append_scale(s) only records K_dev/V_dev; amskv_attend(s)
 * attends to the cache as the previous step left it plus scale s read in place.  Algorithm 1's
 * iteration for scale s (budget test, skip, Algorithm 2's trim, copy of what stays of scale s)
 * comes after that attention.  Whenever its outcome is known before the step runs, the attention
 * launch itself performs it and the iteration is complete when amskv_attend returns: the scale
 * fits the budget untrimmed (it is written behind the cached tokens); or it overflows, on a bf16
 * cache at a step whose (b,h) each belong to one workgroup (at most 256 query tokens at head dim
 * 64, 128 at head dim 128): the kernel then writes Algorithm 2's survivors -- cached tokens that
 * slide toward offset 0 and the kept part of the new scale -- to their new places as they stream
 * through it (a token is only ever written below the place it was read from, by the workgroup
 * that has already read everything below).  If the iteration needs the Eq. 3 score, the
 * similarity kernels and a one-lane kernel that compares the score with theta are enqueued in
 * front of the attention launch, which is handed both outcomes and follows the device's word;
 * the host reads that word (left in pinned host memory by the same kernel, behind one event) when
 * the next call on the layer needs the list.  Not after the last scale of the schedule, whose iteration nobody reads.
 * Otherwise amskv_attend leaves the iteration to the next call that reads or changes
 * the layer's state -- amskv_append_scale, amskv_cache_settle, any query, export -- which
 * enqueues its device work on the stream amskv_attend was given; amskv_cache_reset drops an
 * iteration nobody asked for (after the last step of an image its result is never read).
 * If amskv_attend(s) is not called at all, the next amskv_append_scale or amskv_cache_settle
 * performs the iteration.
 * Where the launch cannot perform the iteration (fp32 caches, steps with more query tokens than
 * one workgroup holds) and the iteration needs the Eq. 3 score, amskv_attend does not wait either:
 * it enqueues the similarity kernels behind the attention -- the last of them leaves the decision
 * in pinned host memory (allocated by amskv_cache_create) -- and an event, and returns.  The call that later
 * performs the iteration waits for that event alone, not for the stream; Algorithm 1 needs the
 * decision only before the next scale is appended, and by then the device has long passed the
 * test when other layers' steps were enqueued in between.
 * K_dev/V_dev of scale s must stay valid and unchanged until the iteration has run: until the
 * work enqueued by the next amskv_append_scale / amskv_cache_settle / query on the layer has
 * finished, or until amskv_cache_reset. */

/* mode = AMSKV_MODE_TOKEN_WINDOW.  The sliding-window and sink-plus-window kept sets that the
 * comparison with other cache strategies (Section 5, the table of SWA / H2O / STA) sets against
 * AMS-KV, at token granularity over the flattened token sequence: budget[l] with c_min == c_max
 * = the window W in tokens and c_cds = the number of sink tokens (0 for a plain sliding window);
 * theta is not used.  After step s the layer holds the first c_cds tokens ever appended and the
 * newest W - c_cds (everything while it fits).  It is the token-budget machinery with one
 * budget and one difference: a scale larger than the window is cut to its newest tokens, not
 * skipped.  Layout, calling order, deferred iteration and buffer lifetimes as in token-budget
 * mode.  (H2O keeps tokens by attention score and is not expressible as a kept set fixed before
 * the step.) */

/* Bytes the arena must have for this configuration: for every layer the K and V regions
 * sized for the largest kept set the policy ever reaches (Section 4.3: capacity is fixed
 * per layer), plus small reduction workspaces for amskv_interscale_similarity and
 * amskv_attention_density.
 * Host only. */
int32_t amskv_cache_required_bytes(int32_t layers, int32_t heads, int32_t head_dim,
                                   const amskv_schedule* schedule, const amskv_policy* policy,
                                   uint64_t* bytes_out);

/* Create the cache (problem statement of Section 4.3: one independent cache per layer,
 * governed by the policy).  arena_dev: device pointer, 256-byte aligned, at least
 * required_bytes long, owned by the caller and kept alive until destroy; it need not be
 * initialised.  arena_dev == NULL creates a plan-only cache: append calls with NULL K/V
 * advance the metadata (layout, bytes held, eviction lists) without touching a GPU, and
 * device calls return AMSKV_ERR_NO_DEVICE_MEMORY.  head_dim must be 64 or 128.
 * The schedule and policy structs are copied.  Host only. */
int32_t amskv_cache_create(int32_t layers, int32_t heads, int32_t head_dim,
                           const amskv_schedule* schedule, const amskv_policy* policy,
                           void* arena_dev, uint64_t arena_bytes, amskv_cache** out);

/* Layout of the caller's per-scale tensors Q, K, V and O (Section 3.1's attention sits between
 * the QKV projection and the output projection, whose activations are token-major).
 *   AMSKV_IO_HEAD_MAJOR (default)  every tensor is [B][H][T_s][D], contiguous
 *   AMSKV_IO_TOKEN_MAJOR           element (b, t, h, d) of a tensor sits at
 *                                  base + ((b*T_s + t) * token_stride + h*D + d) elements
 * with one token stride for Q, one for K and V, one for O (elements; each >= H*D and a multiple
 * of 16 bytes).  A fused projection output [B][T_s][3][H][D] is passed without any copy as
 * Q_dev = p, K_dev = p + H*D, V_dev = p + 2*H*D with q and kv strides 3*H*D; O in [B][T_s][H*D]
 * has stride H*D.  The cache itself stays [B][H][cap][D] per layer, and amskv_cache_export
 * writes head-major.  All device pointers must be 16-byte aligned in either layout.
 * Allowed only while no scale has been appended to any layer (after create or reset), else
 * AMSKV_ERR_ORDER.  Host only. */
int32_t amskv_cache_set_io_layout(amskv_cache* cache, int32_t io_layout, int64_t q_token_stride,
                                  int64_t kv_token_stride, int64_t o_token_stride);

/* Append scale s to layer `layer` (Algorithm 1's append + rolling step, Algorithm 2's
 * eviction at scale granularity): scales that fall outside the policy are evicted, the
 * surviving scales are slid down so the kept set stays contiguous (COMPACT layout), and
 * K_dev/V_dev ([B][H][T_s][D], device) are copied to their slot.  Scales must arrive in
 * order 0,1,2,... per layer (else AMSKV_ERR_ORDER).  The host metadata is updated before
 * the call returns, the device work is asynchronous on `stream`; K_dev/V_dev must stay
 * valid until it has run (longer for a borrowed scale, see borrow_unretained).
 * K_dev == V_dev == NULL updates metadata only. */
int32_t amskv_append_scale(amskv_cache* cache, int32_t layer, int32_t s,
                           const void* K_dev, const void* V_dev, void* stream);

/* Self-attention of generation step s in layer `layer` (Section 3.1: scale s attends to
 * the cached scales and to itself, no mask inside the step):
 *   O[b,h,i,:] = sum_j softmax_j(Q[b,h,i,:].K~[b,h,j,:] * softmax_scale) V~[b,h,j,:]
 * with K~,V~ the concatenation of the resident scales of the layer (scale s included).
 * s must be the scale appended last to this layer (else AMSKV_ERR_ORDER).
 * Q_dev, O_dev: device, [B][H][T_s][D].  bf16: fp32 accumulation and softmax, P rounded
 * to bf16 before the PV product, O rounded to bf16.  Asynchronous on `stream`. */
int32_t amskv_attend(amskv_cache* cache, int32_t layer, int32_t s,
                     const void* Q_dev, void* O_dev, void* stream);

/* Inter-scale similarity of Eq. 3 between scale s and scale s-1 resized bilinearly
 * (half-pixel centres, edge clamp) to the grid of scale s, computed from the cache.
 * Both scales must be resident (else AMSKV_ERR_EVICTED); s >= 1.
 *   cosK_host[h]   mean over (batch, token) of the cosine between k_s[t] and k^_{s-1}[t]
 *   cosV_host[h]   the same for the values, or NULL to skip
 *   sums_host[h*3+{0,1,2}]  sum k.k^, sum |k|^2, sum |k^|^2 over (batch, token, channel)
 *                  of the keys, or NULL; Eq. 3's score is -sqrt(s1 + s2 - 2 s0)
 * Outputs are host arrays of `heads` (resp. 3*heads) floats.  fp32 arithmetic, fixed
 * reduction order (deterministic).  Waits for `stream` before returning. */
int32_t amskv_interscale_similarity(amskv_cache* cache, int32_t layer, int32_t s,
                                    float* cosK_host, float* cosV_host, float* sums_host,
                                    void* stream);

/* The same computation without the wait, for callers that probe many layers: _enqueue only
 * launches the kernels of (layer, s) on `stream` (want_v != 0 includes the values); the sums stay
 * in a per-layer slot inside the arena until the next _enqueue on that layer.  _collect copies
 * the slots of ALL layers to the host with one transfer and one wait for `stream`, and converts
 * them as above: cosK_host[l*H + h], cosV_host[l*H + h] (or NULL), sums_host[(l*H + h)*3 + i]
 * (or NULL).  Layers with nothing enqueued since create / reset, and cosV of a layer enqueued
 * without the values, read NaN.  Same status codes as the call above; all calls of one cache
 * must be ordered on one stream (the partial-sum workspace is shared by the layers). */
int32_t amskv_interscale_similarity_enqueue(amskv_cache* cache, int32_t layer, int32_t s,
                                            int32_t want_v, void* stream);
int32_t amskv_interscale_similarity_collect(amskv_cache* cache, float* cosK_host, float* cosV_host,
                                            float* sums_host, void* stream);

/* For callers that cannot allocate or let the library touch memory it was not handed for this call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The kernels of
 * amskv_interscale_similarity_enqueue with their partial sums in a static device array of the library
 * (2 * AMSKV_STATIC_MAX_UNITS * 4 floats = 512 KB per device, held until the process ends) instead of the
 * arena's workspace, and the result written to the caller's buffer instead of the arena's per-layer slot:
 *   sums_out_dev  device, (want_v ? 2 : 1) * heads * 4 floats, 16-byte aligned: for head h the four sums
 *                 [h*4 + {0,1,2,3}] = sum over (batch, token) of the per-token cosine, sum k.k^, sum |k|^2,
 *                 sum |k^|^2 of the keys, followed (want_v) by the same block for the values.
 *                 cosK[h] = sums[h*4] / (batch * T_s).
 * Calls no allocating routine (the static array's address is looked up once per device, at the first call
 * on it).  batch * heads > AMSKV_STATIC_MAX_UNITS returns AMSKV_ERR_STATIC_LIMIT.  Nothing in the array has
 * to start at zero; every call on a device uses the same array, so calls that overlap in time on one device
 * (different streams, or processes sharing the library image do not count) race and must be ordered by the
 * caller.  Same residency rules and status codes as amskv_interscale_similarity_enqueue otherwise. */
int32_t amskv_interscale_similarity_enqueue_static(amskv_cache* cache, int32_t layer, int32_t s, int32_t want_v,
                                                   float* sums_out_dev, void* stream);

/* Attention density (Section 4.1): of the softmax mass that the queries Q of scale s spread over
 * the keys they attend to, how much lands on each group of keys of layer `layer` -- the groups
 * being the entries of amskv_cache_segments, in that order (whole scales in scale-window mode).
 * Call it where amskv_attend(layer, s) may be called (in token-budget mode before it, since
 * that call ends by trimming the cache).  Outputs, host arrays of heads * AMSKV_MAX_SCALES floats,
 * entry [h * AMSKV_MAX_SCALES + i] for group i < *n_seg, either may be NULL:
 *   mass_host     attention matrix summed over the T_s queries and the keys of the group, mean
 *                 over the batch; the groups of a head add up to T_s
 *   density_host  mass divided by the number of key tokens of the group: the printed definition
 *                 read with A^(j->i) holding one row per query of scale j and one column per key
 *                 of scale i (mass / T_s, the other reading, follows from mass_host)
 * At most AMSKV_MAX_SCALES groups.  bf16 caches: matrix instructions, fp32 arithmetic on the exact
 * bf16 products; fp32 caches: fp32 dot products on the vector ALUs.  Fixed reduction order
 * (deterministic).  Reads Q, the cache and a borrowed scale; writes only its workspace inside the
 * arena.  Waits for `stream` before returning. */
int32_t amskv_attention_density(amskv_cache* cache, int32_t layer, int32_t s, const void* Q_dev,
                                float* density_host, float* mass_host, int32_t* n_seg, void* stream);

/* The same computation without the wait, for callers that analyse many layers: the masses
 * (heads * AMSKV_MAX_SCALES floats, entry [h * AMSKV_MAX_SCALES + i]) are left in mass_out_dev, a
 * caller-owned device buffer (16-byte aligned), in stream order; *n_seg and, if not NULL,
 * tok_len[0 .. *n_seg) (the key tokens of each group: density = mass / tok_len) are host outputs
 * valid on return.  The workspace inside the arena is shared by all layers: calls on one cache
 * must be ordered on one stream. */
int32_t amskv_attention_density_enqueue(amskv_cache* cache, int32_t layer, int32_t s, const void* Q_dev,
                                        float* mass_out_dev, int32_t* n_seg, int32_t* tok_len, void* stream);

/* amskv_attend(layer, s) and the attention density of that step (Section 4.1) in one call: O_dev as
 * amskv_attend leaves it, and in mass_out_dev / *n_seg / tok_len what amskv_attention_density_enqueue
 * would report when called just before -- the groups are the layer's segments as the step's attention
 * sees them, before the step's own bookkeeping (fused append, Algorithm 1's iteration).
 * bf16 caches and steps of more than 32 tokens: the density is a by-product of the attention launch
 * itself -- its kernel keeps, per query row, the sum of exp over the keys of each group next to
 * the softmax statistics it keeps anyway, so Q, K and V are read once and nothing but the per-block
 * partial masses is written beyond O (and the fused append).  O comes out bit-identical to
 * amskv_attend's.  Steps of at most 32 tokens and fp32 caches: the two calls, density first.
 * Status codes and residency rules of amskv_attend; workspace and ordering rule of
 * amskv_attention_density_enqueue. */
int32_t amskv_attend_density(amskv_cache* cache, int32_t layer, int32_t s, const void* Q_dev, void* O_dev,
                             float* mass_out_dev, int32_t* n_seg, int32_t* tok_len, void* stream);

/* Resident segments of a layer, ascending scale id: n_seg entries written to each
 * caller array of at least AMSKV_MAX_SCALES elements.  tok_offset is the position of the
 * segment inside the [cap_l] token axis of the layer's K and V regions, or -1 for a scale
 * that is read in place from the caller's buffers (borrow_unretained).  In token-budget mode
 * the arrays need AMSKV_MAX_SCALES + 2 elements (see amskv_cache_segments).  Host only. */
int32_t amskv_cache_layout(const amskv_cache* cache, int32_t layer, int32_t* n_seg,
                           int32_t* scale_id, int64_t* tok_offset, int32_t* tok_len);

/* Token-granular view of the same list: segment i holds tokens [first_token[i],
 * first_token[i]+tok_len[i]) of scale scale_id[i]; a scale may appear in two segments
 * (Algorithm 2 can keep its head and its tail).  In scale-window mode first_token is 0 and the
 * output equals amskv_cache_layout's.  Arrays hold up to AMSKV_MAX_SCALES + 2 entries.  Host only. */
int32_t amskv_cache_segments(const amskv_cache* cache, int32_t layer, int32_t* n_seg,
                             int32_t* scale_id, int32_t* first_token, int64_t* tok_offset,
                             int32_t* tok_len);

/* Token-budget mode: the budget in force on the layer (c_min, or c_max once expanded);
 * scale-window mode: the layer's capacity in tokens.  Negative amskv_status on error.  Host only. */
int64_t amskv_cache_budget_tokens(const amskv_cache* cache, int32_t layer);

/* Finish whatever the layer still owes for its newest scale without running attention: in
 * token-budget mode Algorithm 1's iteration for that scale, with fuse_append the deferred copy.
 * A no-op when nothing is owed.  On a plan-only cache only the metadata advances. */
int32_t amskv_cache_settle(amskv_cache* cache, int32_t layer, void* stream);

/* Scales dropped by the most recent append to this layer (ascending), for inspection.  In
 * token-budget mode: scales that lost cached tokens, wholly or in part, in the most recent
 * iteration of Algorithm 1 on the layer. */
int32_t amskv_cache_last_evicted(const amskv_cache* cache, int32_t layer, int32_t* n_evicted,
                                 int32_t* scale_id);

/* K+V bytes visible to a layer's attention: 2 * elem * B * H * D * sum of T_k over the resident
 * scales (a borrowed current scale counts only under include_current != 0)
 * (Eq. 4's accounting with its constant written as 2*elem).  include_current == 0 leaves
 * out the newest scale (Algorithm 1 never stores a scale larger than C_max, so the
 * paper's end-of-generation figure excludes it).  Negative status on error.  Host only. */
int64_t amskv_cache_bytes_held(const amskv_cache* cache, int32_t layer, int32_t include_current);

/* Token capacity cap_l of a layer's K (and V) region, or a negative status. */
int64_t amskv_cache_capacity_tokens(const amskv_cache* cache, int32_t layer);

/* Copy the resident scales of a layer, ascending and back to back, into
 * K_out_dev/V_out_dev ([B][H][T_kept][D], device, caller-owned; either may be NULL).
 * For bit-exact checks of slot selection, eviction and compaction.  Asynchronous. */
int32_t amskv_cache_export(const amskv_cache* cache, int32_t layer,
                           void* K_out_dev, void* V_out_dev, void* stream);

/* Forget every appended scale of every layer (metadata only; the arena is not cleared). */
int32_t amskv_cache_reset(amskv_cache* cache);

/* Free the host metadata.  The arena stays the caller's. */
void amskv_cache_destroy(amskv_cache* cache);

/* Static text for a status code. */
const char* amskv_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* AMSKV_H */
