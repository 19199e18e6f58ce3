"""Float64 CPU oracle for the KVCompose prefill-time compression pass.

TEST INFRASTRUCTURE ONLY.  This module exists so that the HIP library can be
checked against the method as the paper defines it.  Only the test-suite, the
smoke check and the benchmark's CPU-baseline leg may import it; the product
path never does, and it shares no code with the HIP path.

Every function is the paper's definition written out step by step in float64,
with no blocking, fusion or reordering, so it can be checked against the paper
by eye.  Indices are 0-based throughout.

Notation (Preliminary and Section 3 of the paper): Lyr layers, Hq query heads,
Hkv KV heads, G = Hq/Hkv, head dimension d, N context tokens, M task
(observation-window) tokens, B = B_total retained composite tokens.

Readings taken where the paper is silent or ambiguous (each is also a library
convention, stated in the C header):

* The M task queries are an input; every query row attends to all N cached
  keys with no mask, and the softmax is normalised over exactly those N keys
  (eq. 3 of the Preliminary: softmax(q K^T / sqrt(d_h)) over the cached keys).
* The GQA reshape Hq -> (Hkv, G) is row-major: query head q = h*G + g
  (Section 3.2.2; the printed group equation lost its h index).
* argsort ties: equal scores keep ascending original index (stable).
* "top-B_total of P" with ties at the threshold: all entries above the
  threshold, then entries equal to it in ascending flat index l*N + k.
* A layer may end with N_l = 0.  No token is force-kept.
* Rows of K', V' are in descending-importance (rank) order, as the final
  selection equations literally index K with idx[:N_l].
* The budget is an integer; B_total = floor((1-r) * Lyr * N) is evaluated by
  the caller.

Variants beyond the default pass (each off unless asked for):

* value-norm weighting (Appendix on value norms, "v-norm"): every entry of the
  attention matrix of query head q is multiplied by the Euclidean norm of the
  value vector of the same token in q's KV head, before any aggregation.
* position order: the retained rows of a head are written in ascending token
  position instead of rank order (the retained *set* is unchanged), so that a
  100 % budget reproduces K and V bit for bit.
* per-layer floor m (the paper does not exclude N_l = 0 and defines no floor;
  this reading): ranks 0..m-1 of every layer are taken first, the rest of the
  budget goes to the top of the remaining pool with the usual tie rule.
* causal tail (a reading for the case where the M task tokens are the last M
  tokens of the context itself, the task-agnostic setting of Section 3.2.1):
  task token m sits at position N-M+m and attends to the cached keys at
  positions <= N-M+m only; its softmax runs over those keys and the other
  entries of its row of A are 0.  Needs N >= M.
* forced retention (not in the paper's method; the attention-sink and
  recent-window conventions its related-work section describes): the first
  keep_first and the last keep_last tokens of the context get the score +inf in
  every head of every layer, so they rank first (ascending position among
  themselves) and are retained whenever the budget allows (B >= Lyr * number of
  forced tokens).
* unstructured selection (Appendix on unstructured eviction): the head
  aggregation is skipped, the pool holds all Lyr*Hkv*N rank-aligned scores,
  the budget counts (head, token) entries and every head keeps its own prefix
  N_{l,h}.  Ties by ascending flat index (l*Hkv + h)*N + k.

Pins (tests/test_oracle_*.py): library softmax in the single-query special
case, closed forms (identical keys), shift/permutation invariants, row-sum
identities, one-hot limit, library stable argsort, brute-force enumeration of
the global selection and of per-head subsets on tiny inputs, budget identities.
"""
from __future__ import annotations

import numpy as np

AGG_MAX = 0
AGG_MEAN = 1


# --------------------------------------------------------------------------
# input widening (the oracle's own; the HIP path consumes the raw bits)
# --------------------------------------------------------------------------
def widen(x: np.ndarray) -> np.ndarray:
    """Exact float64 value of a float32 array or of bf16 bit patterns (uint16)."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def _agg(x: np.ndarray, op: int, axis: int) -> np.ndarray:
    if op == AGG_MAX:
        return x.max(axis=axis)
    if op == AGG_MEAN:
        return x.mean(axis=axis)
    raise ValueError("unknown aggregation operator")


# --------------------------------------------------------------------------
# Section 3.2.2: attention collection and aggregation
# --------------------------------------------------------------------------
def attention(q_rows: np.ndarray, keys: np.ndarray, scale: float,
              causal_tail: bool = False) -> np.ndarray:
    """A[m, c] = softmax_c(q_m . k_c * scale) for M query rows and N cached keys.

    Preliminary eq. 3 applied to each task token; the softmax runs over the N
    cached keys only.  causal_tail: row m only sees keys c <= N - M + m.
    """
    s = (q_rows @ keys.T) * scale                     # [M, N]
    if causal_tail:
        m, n = s.shape
        if n < m:
            raise ValueError("causal tail needs N >= M")
        hidden = np.arange(n)[None, :] > (n - m + np.arange(m))[:, None]
        s = np.where(hidden, -np.inf, s)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def score_layer(q, k, *, agg_task=AGG_MAX, agg_group=AGG_MEAN, add_head_mean=True,
                scale=None, v=None, causal_tail=False) -> np.ndarray:
    """S[h, c] for one layer of one sequence.

    q: [Hq, M, d], k: [Hkv, N, d] (float64).  Follows, in order, the three
    equations of Section 3.2.2: aggregation over task tokens (eq. 14),
    aggregation over the query heads of a KV group (eq. 15) and the head-mean
    augmentation that follows them.

    v: optional [Hkv, N, d] (float64).  When given, the attention matrix of
    every query head is replaced by the weighted matrix of the value-norm
    appendix (v-norm variant): A^(w)[m, c] = A[m, c] * ||V[h, c, :]||_2 with h
    the KV head of the query head.
    """
    hq, m, d = q.shape
    hkv, n, _ = k.shape
    g = hq // hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    s_task = np.empty((hq, n))
    for qh in range(hq):
        a = attention(q[qh], k[qh // g], scale, causal_tail)   # [M, N]: A^(l, qh, c, m)
        if v is not None:
            a = a * np.sqrt((v[qh // g] * v[qh // g]).sum(axis=1))[None, :]   # A^(w)
        s_task[qh] = _agg(a, agg_task, axis=0)        # eq. 14
    s_group = _agg(s_task.reshape(hkv, g, n), agg_group, axis=1)   # eq. 15
    if add_head_mean:
        return s_group + s_group.sum(axis=0, keepdims=True) / hkv  # augmentation
    return s_group


def force_keep(s: np.ndarray, keep_first: int, keep_last: int) -> np.ndarray:
    """Scores with the first keep_first and the last keep_last tokens set to +inf."""
    n = s.shape[-1]
    if keep_first < 0 or keep_last < 0:
        raise ValueError("keep_first / keep_last must be >= 0")
    if keep_first == 0 and keep_last == 0:
        return s
    s = s.copy()
    s[..., :min(keep_first, n)] = np.inf
    s[..., max(n - keep_last, 0):] = np.inf
    return s


# --------------------------------------------------------------------------
# Section 3.3: composite tokens
# --------------------------------------------------------------------------
def head_rank(s: np.ndarray):
    """idx[..., k] = position with the k-th largest score (ties: lower index
    first) and S'[..., k] = S[..., idx[..., k]]  (Section 3.3: the per-head
    descending argsort, eq. 17, and the rank-aligned scores defined after it).

    Written as a plain loop-free definition: sort pairs (-score, index)
    lexicographically.
    """
    s = np.asarray(s)
    n = s.shape[-1]
    flat = s.reshape(-1, n)
    idx = np.empty(flat.shape, dtype=np.int64)
    pos = np.arange(n)
    for r in range(flat.shape[0]):
        idx[r] = np.lexsort((pos, -flat[r]))          # primary key -score, then index
    s_sorted = np.take_along_axis(flat, idx, axis=1)
    return idx.reshape(s.shape), s_sorted.reshape(s.shape)


def composite(s_sorted: np.ndarray, agg_head=AGG_MEAN) -> np.ndarray:
    """I[k] = Agg_h S'[h, k] for one layer: the composite importance score that
    Section 3.3 defines right after the rank-aligned scores.  s_sorted: [Hkv, N]."""
    return _agg(np.asarray(s_sorted, dtype=np.float64), agg_head, axis=0)


def global_select(i_all: np.ndarray, budget: int, min_per_layer: int = 0):
    """Per-layer lengths from the global pool (Section 3.3, pool / budget /
    N_l equations).

    i_all: [Lyr, N].  The pool P holds all Lyr*N composite scores; the top
    ``budget`` of them are taken (ties by ascending flat index l*N + k) and
    N_l counts how many of the taken entries lie in layer l.  Returns
    (lengths int64 [Lyr], tau) with tau the smallest taken score (None when
    budget == 0).

    min_per_layer = m > 0 (per-layer floor, a reading: the paper defines
    none): ranks 0..min(m, N)-1 of every layer are taken unconditionally and
    only the other pool entries compete for the rest of the budget; tau is
    then the smallest score taken in that competition (None if nothing is
    left to compete for).

    The rows of i_all may as well be (layer, head) pairs holding rank-aligned
    per-head scores: that is the unstructured variant's pool.
    """
    i_all = np.asarray(i_all)
    lyr, n = i_all.shape
    floor = min(int(min_per_layer), n)
    if floor < 0 or not lyr * floor <= budget <= lyr * n:
        raise ValueError("budget out of range")
    pool = i_all.reshape(-1)
    flat = np.arange(pool.size)
    free = flat[(flat % n) >= floor]                  # entries that compete
    order = free[np.lexsort((free, -pool[free]))]
    taken = order[:budget - lyr * floor]
    lengths = floor + np.bincount(taken // n, minlength=lyr).astype(np.int64)
    tau = pool[taken[-1]] if taken.size > 0 else None
    return lengths, tau


def gather(x: np.ndarray, idx: np.ndarray, n_keep: int, position_order: bool = False) -> np.ndarray:
    """X'[h, k, :] = X[h, idx[h, k], :], k < n_keep (final selection equations).

    position_order: the same retained set idx[h, :n_keep] of every head, but
    written in ascending token position."""
    hkv = x.shape[0]
    out = np.empty((hkv, n_keep) + x.shape[2:], dtype=x.dtype)
    for h in range(hkv):
        rows = idx[h, :n_keep]
        out[h] = x[h, np.sort(rows) if position_order else rows]
    return out


def gather_heads(x: np.ndarray, idx: np.ndarray, n_keep, position_order: bool = False) -> list:
    """Unstructured variant: head h keeps its own prefix idx[h, :n_keep[h]].
    Returns a list of Hkv arrays [n_keep[h], d]."""
    out = []
    for h in range(x.shape[0]):
        rows = idx[h, :int(n_keep[h])]
        out.append(x[h, np.sort(rows) if position_order else rows])
    return out


# --------------------------------------------------------------------------
# whole pass for one sequence
# --------------------------------------------------------------------------
def compress(q_layers, k_layers, v_layers, budget: int, *, agg_task=AGG_MAX,
             agg_group=AGG_MEAN, agg_head=AGG_MEAN, add_head_mean=True, scale=None,
             value_norm=False, position_order=False, min_per_layer=0, unstructured=False,
             causal_tail=False, keep_first=0, keep_last=0):
    """Run the pass on one sequence.

    q_layers[l]: [Hq, M, d]; k_layers[l], v_layers[l]: [Hkv, N, d]; any of
    float32 / float64 / bf16 bits (uint16).  K' and V' keep the input dtype
    (bit copies).  Returns a dict with every intermediate.

    unstructured: budget counts (head, token) entries; "lengths" is [Lyr, Hkv],
    "I" is None and K_out[l] / V_out[l] are lists of per-head arrays.
    """
    lyr = len(k_layers)
    s_all, idx_all, ssorted_all, i_all = [], [], [], []
    for l in range(lyr):
        s = score_layer(widen(q_layers[l]), widen(k_layers[l]), agg_task=agg_task,
                        agg_group=agg_group, add_head_mean=add_head_mean, scale=scale,
                        v=widen(v_layers[l]) if value_norm else None, causal_tail=causal_tail)
        s = force_keep(s, keep_first, keep_last)
        idx, s_sorted = head_rank(s)
        s_all.append(s)
        idx_all.append(idx)
        ssorted_all.append(s_sorted)
        i_all.append(composite(s_sorted, agg_head))
    i_all = np.stack(i_all)
    if unstructured:
        s3 = np.stack(ssorted_all)                                   # [Lyr, Hkv, N]
        hkv, n = s3.shape[1], s3.shape[2]
        flat_len, tau = global_select(s3.reshape(lyr * hkv, n), budget, min_per_layer)
        lengths = flat_len.reshape(lyr, hkv)
        k_out = [gather_heads(np.asarray(k_layers[l]), idx_all[l], lengths[l], position_order)
                 for l in range(lyr)]
        v_out = None
        if v_layers is not None:
            v_out = [gather_heads(np.asarray(v_layers[l]), idx_all[l], lengths[l], position_order)
                     for l in range(lyr)]
        return {
            "S": np.stack(s_all), "idx": np.stack(idx_all), "S_sorted": s3,
            "I": None, "tau": tau, "lengths": lengths, "K_out": k_out, "V_out": v_out,
        }
    lengths, tau = global_select(i_all, budget, min_per_layer)
    k_out = [gather(np.asarray(k_layers[l]), idx_all[l], int(lengths[l]), position_order)
             for l in range(lyr)]
    v_out = None
    if v_layers is not None:
        v_out = [gather(np.asarray(v_layers[l]), idx_all[l], int(lengths[l]), position_order)
                 for l in range(lyr)]
    return {
        "S": np.stack(s_all), "idx": np.stack(idx_all), "S_sorted": np.stack(ssorted_all),
        "I": i_all, "tau": tau, "lengths": lengths, "K_out": k_out, "V_out": v_out,
    }
