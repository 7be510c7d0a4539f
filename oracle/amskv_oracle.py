"""CPU oracle for the AMS-KV hot path (arxiv 2511.16047).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, fp64 statement of what
the GPU library must compute.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does.  It shares no code with
the HIP library: the kept-set rule, the offsets, the mask, the softmax, the bilinear
resize and the similarity sums are all written out again here.

Notation (Section "Preliminaries" and Section 4.3 of the paper): a schedule of S
scales, scale s being an h_s x w_s grid of T_s = h_s*w_s tokens stored row-major;
global token index g = start_s + r*w_s + c.  A layer policy is the triple
(n_condensed c, window w, keep_all).

Readings taken where the paper is silent or ambiguous (each is repeated at the
function it affects):
  * eviction is scale-granular: a scale is either wholly kept or wholly dropped
    (the prose of Section 4.3 speaks of evicting whole scales; the token slicing of
    Algorithm 2 is modelled separately in `clru` / `alg1_cache_trace`, and the
    token windows of the comparison policies in `token_window_cache`);
  * at step s the queries of scale s see the condensed scales {0..c-1}, the w scales
    that precede s, and s itself, all clipped to [0, s];
  * softmax scale defaults to 1/sqrt(D), no bias;
  * "2D interpolation" (Eq. 3) is bilinear with half-pixel centres and edge clamping;
  * the similarity is reported as a cosine (mean over tokens) together with the three
    flattened sums from which Eq. 3's negative L2 distance follows.

Pins (tests/test_oracle_pins.py): closed-form kept-token counts, set enumeration on
tiny schedules, equality with plain block-causal attention when the window covers
every scale, library attention on the gathered kept keys, rows of P summing to one,
O = V at scale 0, NaN-poisoned evicted scales, pure-Python triple loops on a 3-scale
schedule, library bilinear resize, affine-ramp reproduction, cos = +-1 cases, and the
token-id sets of Algorithms 1 and 2 (hand-derived traces, closed-form masks), the token
windows (hand trace, token-by-token queue, the cases that reduce to Algorithm 1 and to the
block-causal mask), and
for the attention density: mass summing to T_s, an element-by-element brute force, the
uniform and the one-dominant-key cases.  No function here is "parity unpinned";
the paper's printed GB and percent figures are unpinned (its Tables 3 and 5 disagree
with each other and with Eq. 4) and are quoted, never asserted.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

Policy = Tuple[int, int, bool]  # (n_condensed, window, keep_all)


# --------------------------------------------------------------------------- schedule
def scale_tokens(side_h: Sequence[int], side_w: Sequence[int]) -> List[int]:
    """T_s = h_s * w_s (Section 3.1: each scale r_k is an h_k x w_k token map)."""
    return [int(h) * int(w) for h, w in zip(side_h, side_w)]


def scale_starts(tokens: Sequence[int]) -> List[int]:
    """start_s = sum_{k<s} T_k: where scale s begins in the whole token sequence."""
    out, acc = [], 0
    for t in tokens:
        out.append(acc)
        acc += int(t)
    return out


def scale_of_token(tokens: Sequence[int]) -> np.ndarray:
    """scale id of every global token index (lookup table over the whole sequence)."""
    return np.concatenate([np.full(int(t), s, dtype=np.int64) for s, t in enumerate(tokens)])


# --------------------------------------------------------------------------- policy
def visible(policy: Policy, q_scale: int, k_scale: int) -> bool:
    """May a query of scale q_scale read keys of scale k_scale?

    Block-causal next-scale prediction (Eq. 2: scale k conditions on scales < k, and
    tokens of one scale are produced together, so they see each other) restricted by
    the AMS-KV taxonomy of Section 4.1/4.3: condensed scales (the first c) stay,
    local scales (the w most recent before the current one) roll, the rest are gone.
    """
    c, w, keep_all = policy
    if k_scale > q_scale:
        return False
    if keep_all:
        return True
    return k_scale < c or (q_scale - k_scale) <= w


def kept_scales(policy: Policy, s: int) -> List[int]:
    """Ascending ids of the scales resident after scale s has been appended."""
    return [k for k in range(s + 1) if visible(policy, s, k)]


def evicted_scales(policy: Policy, s: int) -> List[int]:
    """Scales resident after step s-1 that are no longer resident after step s."""
    if s == 0:
        return []
    before = set(kept_scales(policy, s - 1))
    after = set(kept_scales(policy, s))
    return sorted(before - after)


def stored_scales(policy: Policy, s: int, n_scales: int) -> List[int]:
    """Scales that occupy cache memory after step s when only scales a LATER step reads are
    stored (Algorithm 1 appends a scale for the benefit of the following iterations; a scale
    no later step sees -- the last one of the schedule, or any non-condensed scale under a
    zero window -- is used by its own step's attention and never written to the cache)."""
    out = []
    for k in kept_scales(policy, s):
        read_later = any(visible(policy, later, k) for later in range(k + 1, n_scales))
        if read_later:
            out.append(k)
    return out


def stored_capacity(tokens: Sequence[int], policy: Policy) -> int:
    n = len(tokens)
    return max(sum(int(tokens[k]) for k in stored_scales(policy, s, n)) for s in range(n))


def kept_token_count(tokens: Sequence[int], policy: Policy, s: int) -> int:
    return sum(int(tokens[k]) for k in kept_scales(policy, s))


def segment_offsets(tokens: Sequence[int], policy: Policy, s: int) -> List[int]:
    """Token offset of every kept scale inside the compacted cache (exclusive prefix sum)."""
    offs, acc = [], 0
    for k in kept_scales(policy, s):
        offs.append(acc)
        acc += int(tokens[k])
    return offs


def cache_capacity(tokens: Sequence[int], policy: Policy) -> int:
    """Largest number of tokens the layer ever holds over the whole schedule."""
    return max(kept_token_count(tokens, policy, s) for s in range(len(tokens)))


def bytes_held(tokens: Sequence[int], policy: Policy, s: int, batch: int, heads: int,
               head_dim: int, elem_bytes: int, include_current: bool = True) -> int:
    """K+V bytes resident in one layer after step s.

    Same accounting as Eq. 4 (Appendix D) with the per-element constant written as
    2*elem_bytes (K and V, literal batch).  include_current=False leaves the newest
    scale out, which is how Algorithm 1 counts the last step (it never stores a scale
    larger than C_max).
    """
    ks = kept_scales(policy, s)
    if not include_current:
        ks = [k for k in ks if k != s]
    return 2 * elem_bytes * batch * heads * head_dim * sum(int(tokens[k]) for k in ks)


def kv_mem_saving_eq4(tokens: Sequence[int], batch: int, heads: int, head_dim: int,
                      n_layers: int, scales_cd: Sequence[int], n_cd: int,
                      scales_ce: Sequence[int], n_ce: int, bytes_per_pair: float = 16.0) -> float:
    """Eq. 4 (Appendix D), in MB: c*B*H*D/1024^2 * [sum_S T*N - sum_CD T*N_CD - sum_CE T*N_CE]."""
    all_t = sum(int(t) for t in tokens)
    cd_t = sum(int(tokens[k]) for k in scales_cd)
    ce_t = sum(int(tokens[k]) for k in scales_ce)
    return bytes_per_pair * batch * heads * head_dim / 1024.0 ** 2 * (
        all_t * n_layers - cd_t * n_cd - ce_t * n_ce)


# --------------------------------------------------------------------------- mask + attention
def allow_mask(tokens: Sequence[int], policy: Policy) -> np.ndarray:
    """Explicit T x T boolean mask over the whole sequence: allow[q, k]."""
    st = scale_starts(tokens)
    n = sum(int(t) for t in tokens)
    allow = np.zeros((n, n), dtype=bool)
    for q_scale in range(len(tokens)):
        for k_scale in range(len(tokens)):
            if visible(policy, q_scale, k_scale):
                allow[st[q_scale]: st[q_scale] + int(tokens[q_scale]),
                      st[k_scale]: st[k_scale] + int(tokens[k_scale])] = True
    return allow


def masked_attention(q_all: np.ndarray, k_all: np.ndarray, v_all: np.ndarray,
                     allow: np.ndarray, softmax_scale: float | None = None,
                     return_probs: bool = False):
    """Softmax attention over the whole sequence with an explicit mask, fp64.

    q_all, k_all, v_all: [..., T, D].  Every scale's rows are computed at once; the
    result for generation step s is rows start_s .. start_s+T_s-1.
    """
    q = np.asarray(q_all, dtype=np.float64)
    k = np.asarray(k_all, dtype=np.float64)
    v = np.asarray(v_all, dtype=np.float64)
    d = q.shape[-1]
    sigma = 1.0 / math.sqrt(d) if not softmax_scale else float(softmax_scale)
    sc = np.matmul(q, np.swapaxes(k, -1, -2)) * sigma
    sc = np.where(allow, sc, -np.inf)
    sc = sc - sc.max(axis=-1, keepdims=True)
    p = np.exp(sc)
    p = p / p.sum(axis=-1, keepdims=True)
    o = np.matmul(p, v)
    return (o, p) if return_probs else o


def attend_step(q_scales: Sequence[np.ndarray], k_scales: Sequence[np.ndarray],
                v_scales: Sequence[np.ndarray], tokens: Sequence[int], policy: Policy,
                s: int, softmax_scale: float | None = None) -> np.ndarray:
    """Output rows of generation step s, [..., T_s, D] (fp64).

    Builds the whole-sequence K, V and mask up to scale s (later scales cannot be seen by
    scale s, so leaving them out changes nothing) and evaluates the rows of scale s.
    """
    toks = list(tokens[: s + 1])
    k_all = np.concatenate([np.asarray(x, dtype=np.float64) for x in k_scales[: s + 1]], axis=-2)
    v_all = np.concatenate([np.asarray(x, dtype=np.float64) for x in v_scales[: s + 1]], axis=-2)
    allow = allow_mask(toks, policy)
    st = scale_starts(toks)[s]
    # only the query rows of scale s are wanted: take those rows of Q and of the mask
    return masked_attention(np.asarray(q_scales[s], dtype=np.float64), k_all, v_all,
                            allow[st: st + toks[s], :], softmax_scale)


def attend_all_steps(q_scales: Sequence[np.ndarray], k_scales: Sequence[np.ndarray],
                     v_scales: Sequence[np.ndarray], tokens: Sequence[int], policy: Policy,
                     softmax_scale: float | None = None) -> List[np.ndarray]:
    """Every generation step at once: one masked attention over the whole sequence, then the
    rows of each scale.  Same numbers as attend_step(s) for every s."""
    q_all = np.concatenate([np.asarray(x, dtype=np.float64) for x in q_scales], axis=-2)
    k_all = np.concatenate([np.asarray(x, dtype=np.float64) for x in k_scales], axis=-2)
    v_all = np.concatenate([np.asarray(x, dtype=np.float64) for x in v_scales], axis=-2)
    o = masked_attention(q_all, k_all, v_all, allow_mask(tokens, policy), softmax_scale)
    st = scale_starts(tokens)
    return [o[..., st[s]: st[s] + int(tokens[s]), :] for s in range(len(tokens))]


# --------------------------------------------------------------------------- cache contents
def cache_contents(x_scales: Sequence[np.ndarray], policy: Policy, s: int) -> np.ndarray:
    """Compacted cache after step s: kept scales, ascending, concatenated on the token axis.

    x_scales[k] is [B, H, T_k, D] of any dtype (bit patterns are carried unchanged).
    """
    return np.concatenate([x_scales[k] for k in kept_scales(policy, s)], axis=-2)


# --------------------------------------------------------------------------- Eq. 3 similarity
def bilinear_upsample(x: np.ndarray, h_in: int, w_in: int, h_out: int, w_out: int) -> np.ndarray:
    """Resize [..., h_in*w_in, D] token grids to [..., h_out*w_out, D], fp64.

    Half-pixel centres: src = (dst + 0.5) * in/out - 0.5, clamped to [0, in-1]; the two
    neighbours are floor(src) and min(floor(src)+1, in-1).  Rows, then columns.
    """
    x = np.asarray(x, dtype=np.float64)
    lead = x.shape[:-2]
    d = x.shape[-1]
    g = x.reshape(lead + (h_in, w_in, d))

    def taps(n_in, n_out):
        i0 = np.zeros(n_out, dtype=np.int64)
        i1 = np.zeros(n_out, dtype=np.int64)
        lam = np.zeros(n_out, dtype=np.float64)
        for j in range(n_out):
            src = (j + 0.5) * n_in / n_out - 0.5
            src = min(max(src, 0.0), n_in - 1.0)
            a = int(math.floor(src))
            i0[j] = a
            i1[j] = min(a + 1, n_in - 1)
            lam[j] = src - a
        return i0, i1, lam

    r0, r1, lr = taps(h_in, h_out)
    c0, c1, lc = taps(w_in, w_out)
    rows = g[..., r0, :, :] * (1.0 - lr)[:, None, None] + g[..., r1, :, :] * lr[:, None, None]
    out = rows[..., :, c0, :] * (1.0 - lc)[:, None] + rows[..., :, c1, :] * lc[:, None]
    return out.reshape(lead + (h_out * w_out, d))


def interscale_similarity(x_s: np.ndarray, x_prev: np.ndarray, side_s: Tuple[int, int],
                          side_prev: Tuple[int, int]):
    """Similarity between scale s and the up-sampled scale s-1 (Eq. 3), per head.

    x_s: [B, H, T_s, D], x_prev: [B, H, T_{s-1}, D].  Returns
      cos[H]      mean over (batch, token) of <a_t, b_t> / max(|a_t| |b_t|, 1e-12),
      sums[H, 3]  sum a.b, sum |a|^2, sum |b|^2 over (batch, token, channel),
    with a = x_s and b = bilinear(x_prev).  Eq. 3's score for a head is
    -sqrt(sums[1] + sums[2] - 2 sums[0]).
    """
    a = np.asarray(x_s, dtype=np.float64)
    b = bilinear_upsample(x_prev, side_prev[0], side_prev[1], side_s[0], side_s[1])
    dot = (a * b).sum(-1)
    na = np.sqrt((a * a).sum(-1))
    nb = np.sqrt((b * b).sum(-1))
    cos_t = dot / np.maximum(na * nb, 1e-12)
    cos = cos_t.mean(axis=(0, 2))
    sums = np.stack([dot.sum(axis=(0, 2)), (a * a).sum(axis=(0, 2, 3)), (b * b).sum(axis=(0, 2, 3))], axis=-1)
    return cos, sums


def neg_l2_from_sums(sums: np.ndarray) -> np.ndarray:
    """Eq. 3: S = -||k_i - k^_{i-1}||_2, from the three flattened sums."""
    s = np.asarray(sums, dtype=np.float64)
    return -np.sqrt(np.maximum(s[..., 1] + s[..., 2] - 2.0 * s[..., 0], 0.0))


# --------------------------------------------------------------------------- Algorithms 1 and 2 at token granularity
# Stated here as what the two algorithms define rather than as their listings: the cache of a layer
# is a SET of global token ids (ids grow with arrival time, so "oldest" = smallest id), Algorithm 2
# is a selection rule on such a set, and one iteration of Algorithm 1 is three predicates on the
# sizes involved followed by that selection.
def clru(entries: Sequence[int], c_bgt: int, c_cds: int) -> List[int]:
    """What Algorithm 2 leaves of a set of cached token ids under the budget c_bgt: everything if
    it fits, otherwise the c_cds oldest ids (the condensed part) and the c_bgt - c_cds newest."""
    ids = np.sort(np.asarray(list(entries), dtype=np.int64))
    if ids.size <= c_bgt:
        return ids.tolist()
    rank = np.arange(ids.size)
    keep = (rank < c_cds) | (rank >= ids.size - (c_bgt - c_cds))
    return ids[keep].tolist()


def alg1_cache_trace(tokens: Sequence[int], c_min: int, c_max: int, c_cds: int,
                     below_theta) -> List[Tuple[List[int], int]]:
    """The cache Algorithm 1 (Section 4.3) holds after every scale, token-granular.

    Definition used.  With cache C and budget b before scale i (T_i tokens, ids I_i):
      * the scale is a candidate only if T_i <= C_max;
      * it overflows if |C| + T_i > b;
      * an overflowing candidate met while b = C_min asks the similarity test of Eq. 3, and a
        positive answer raises b to C_max for every later scale too;
      * the scale is admitted if it is a candidate and, when it overflows, T_i <= b (after the raise);
      * C becomes Algorithm 2's selection from C u I_i if admitted, and stays as it is otherwise.
    below_theta: a sequence of bools per scale, or a callable (i, cached ids before) -> bool that
    is called exactly when the test is asked.
    Returns, per scale, (sorted cached ids after it, budget in force after it).
    """
    starts = scale_starts(tokens)
    held = np.zeros(0, dtype=np.int64)
    budget = c_min
    out: List[Tuple[List[int], int]] = []
    for i, t in enumerate(int(x) for x in tokens):
        candidate = t <= c_max
        overflows = candidate and held.size + t > budget
        if overflows and budget == c_min:
            answer = below_theta(i, held.tolist()) if callable(below_theta) else below_theta[i]
            if answer:
                budget = c_max
        if candidate and (not overflows or t <= budget):
            held = np.asarray(clru(np.concatenate([held, starts[i] + np.arange(t)]), budget, c_cds), dtype=np.int64)
        out.append((held.tolist(), budget))
    return out


def alg1_allow_mask(tokens: Sequence[int], trace: Sequence[Tuple[List[int], int]]) -> np.ndarray:
    """T x T mask of the token-granular reading of Algorithm 1 (Section 4.3): the tokens of
    scale i attend to what the cache held after iteration i-1 and to their own scale (the
    paper never says when attention runs; this reading makes C_min = "condensed plus the
    penultimate scale" of Section 5 what the final step sees)."""
    st = scale_starts(tokens)
    n = sum(int(t) for t in tokens)
    allow = np.zeros((n, n), dtype=bool)
    for i, t in enumerate(tokens):
        rows = slice(st[i], st[i] + int(t))
        allow[rows, st[i]: st[i] + int(t)] = True
        if i > 0:
            allow[rows, np.asarray(trace[i - 1][0], dtype=np.int64)] = True
    return allow


# --------------------------------------------------------------------------- token windows (SWA / STA kept sets)
def token_window_cache(tokens: Sequence[int], window: int, n_sink: int = 0) -> List[List[int]]:
    """Cached token ids after every step under a fixed budget of `window` tokens over the flattened
    token sequence: the sliding-window (n_sink = 0) and sink-plus-window kept sets that the
    comparison with other cache strategies (Section 5, table of SWA / H2O / STA at a fixed
    compression ratio) sets against AMS-KV.  Reading taken, the paper giving no definition for
    next-scale prediction: after step i the cache holds, of all tokens of scales 0..i in order of
    arrival, the first n_sink and the most recent window - n_sink (all of them while they fit);
    a scale larger than the window is cut, never skipped."""
    assert 0 <= n_sink <= window
    starts = scale_starts(tokens)
    out = []
    for i, t in enumerate(tokens):
        seen = starts[i] + int(t)
        if seen <= window:
            out.append(list(range(seen)))
        else:
            out.append(list(range(n_sink)) + list(range(seen - (window - n_sink), seen)))
    return out


def token_window_allow_mask(tokens: Sequence[int], window: int, n_sink: int = 0) -> np.ndarray:
    """T x T mask of that policy: a query of scale i sees its own scale and what the cache held
    after step i-1, written as a predicate on (query id, key id) alone."""
    assert 0 <= n_sink <= window
    sc = scale_of_token(tokens)
    st = np.asarray(scale_starts(tokens), dtype=np.int64)
    n = sc.size
    key = np.arange(n)[None, :]
    own_start = st[sc][:, None]                      # first token of the query's scale = tokens seen before it
    same = sc[:, None] == sc[None, :]
    past = key < own_start
    fits = own_start <= window
    recent = key >= own_start - (window - n_sink)
    return same | (past & (fits | recent | (key < n_sink)))


# --------------------------------------------------------------------------- attention density
def attention_density(q_s: np.ndarray, k_all: np.ndarray, allow_rows: np.ndarray,
                      pieces: Sequence[Tuple[int, int]], softmax_scale: float | None = None):
    """Attention density of Section 4.1 for the queries of one scale.

    q_s: [B, H, T_s, D] queries of the scale being generated; k_all: [B, H, T, D] keys of the
    whole sequence; allow_rows: [T_s, T] mask rows of those queries; pieces: (first global token,
    length) of each group of keys (a scale, or the part of a scale that is cached).
    Returns (density[H, n_pieces], mass[H, n_pieces]): mass is the attention matrix summed over
    the queries of the scale and the keys of the piece, averaged over the batch; density divides
    it by the number of key tokens of the piece.  Reading of the printed definition: A^(j->i) has
    one row per query of scale j and one column per key of scale i, so T_i counts key tokens and
    the density is attention mass per cached token.  mass / T_s (the other reading) follows from
    the second output.
    """
    q = np.asarray(q_s, dtype=np.float64)
    zeros_v = np.zeros(np.asarray(k_all).shape, dtype=np.float64)
    _, p = masked_attention(q, k_all, zeros_v, allow_rows, softmax_scale, return_probs=True)
    mass = np.stack([p[..., a: a + n].sum(axis=(-1, -2)) for a, n in pieces], axis=-1)  # [B, H, n_pieces]
    mass = mass.mean(axis=0)
    dens = mass / np.asarray([n for _, n in pieces], dtype=np.float64)
    return dens, mass
