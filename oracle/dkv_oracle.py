"""CPU oracle for DynamicKV's prefill-time KV compression (arxiv 2412.14838).

TEST INFRASTRUCTURE ONLY.  This is the plain, slow reference the HIP kernels are
checked against.  It shares no code with the HIP path and nothing in the
product may import it; only the tests, the smoke check and the benchmark's
cpu_baseline leg call it.

The method is a heuristic, so the oracle takes the steps of Algorithm 1
("DynamicKV in Prefill Phase") in the paper's order, one sequence at a time
(prefill is per sample, Section 4.3 Q1), in float64.  Pooled scores are rounded
once to float32 (step O5) so that every later, integer-valued decision is a pure
function of float32 values - the precision the kernels take those decisions in.

Notation (paper -> here): L layers; H -> Hq query heads / Hkv KV heads,
G = Hq // Hkv; d_k -> d; S sequence length; ws -> w; prefix length S' = S - w;
(wt - ws) -> mean_budget; B^l = (wt - ws) * r_max -> layer_max;
B = (wt - ws) * L -> global budget; m -> interval.

Readings where the paper is silent or garbled (each one is a decision shared
with the kernels and listed in the design notes):
  * softmax scale 1/sqrt(d) (Eq. 1; the algorithm listing omits it);
  * causal mask inside the window: window query i sits at position S - w + i;
  * window rows are summed (row_scale = 1; 1/w gives the listing's mean);
  * GQA: the G query heads of a KV head are summed before pooling;
  * pooling = max, kernel P, stride 1, same length, taken over the prefix only;
  * ties in every top-k go to the lower (flat) index;
  * flat index -> layer by integer division with Hkv * S' (the listing's
    divisor is garbled);
  * the normalisation of the counts cancels in t / max, and both int() steps
    are exact integer floors;
  * truncation never grows a layer: n_i <- min(n_i, Z'_i).
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# Eq. 1-2 / Algorithm 1 "A^l_h <- softmax(...).mean(dim=-2).pooling(dim=-1)"
# --------------------------------------------------------------------------
def window_logits(q_win: np.ndarray, k: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """O1+O2: x[g, i, s] = scale * <q_win[g, i], k[g // G, s]>, causally masked.

    q_win [Hq, w, d], k [Hkv, S, d] -> x [Hq, w, S] float64 (Eq. 1 numerator).
    """
    q = np.asarray(q_win, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    Hq, w, d = q.shape
    Hkv, S, _ = kk.shape
    assert Hq % Hkv == 0 and S >= w
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    x = np.empty((Hq, w, S), dtype=np.float64)
    for g in range(Hq):
        x[g] = scale * (q[g] @ kk[g // G].T)
    # window query i is the token at position S - w + i and sees keys s <= S - w + i
    pos = np.arange(S)[None, :]
    own = (S - w + np.arange(w))[:, None]
    x[:, pos > own] = -np.inf
    return x


def softmax_rows(x: np.ndarray) -> np.ndarray:
    """O3: softmax over the key axis (Eq. 1)."""
    m = x.max(axis=-1, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=-1, keepdims=True)


def window_sum(p: np.ndarray, Hkv: int, row_scale: float = 1.0) -> np.ndarray:
    """O4: a[h, s] = row_scale * sum over the G heads of KV head h and the w window rows."""
    Hq, w, S = p.shape
    G = Hq // Hkv
    return row_scale * p.reshape(Hkv, G * w, S).sum(axis=1)


def max_pool_prefix(a: np.ndarray, w: int, P: int) -> np.ndarray:
    """O5: A[h, s] = max_{|j - s| <= (P-1)/2, 0 <= j < S'} a[h, j] for s in [0, S'), as float32 (Eq. 2)."""
    assert P % 2 == 1 and P >= 1
    Hkv, S = a.shape
    Sp = S - w
    half = (P - 1) // 2
    pre = a[:, :Sp]
    out = np.empty((Hkv, Sp), dtype=np.float64)
    for s in range(Sp):
        lo, hi = max(0, s - half), min(Sp - 1, s + half)
        out[:, s] = pre[:, lo:hi + 1].max(axis=1)
    return out.astype(np.float32)


def score_window(q_win: np.ndarray, k: np.ndarray, P: int, scale: Optional[float] = None,
                 row_scale: float = 1.0) -> np.ndarray:
    """Steps O1-O5 for one layer of one sequence -> A^l [Hkv, S'] float32."""
    Hq, w, _ = q_win.shape
    Hkv = k.shape[0]
    p = softmax_rows(window_logits(q_win, k, scale))
    a = window_sum(p, Hkv, row_scale)
    return max_pool_prefix(a, w, P)


def row_lse(q_win: np.ndarray, k: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """Natural-log normaliser of every window row: lse[g, i] = log sum_s exp(x[g, i, s]) over the visible keys.

    This is the denominator of Eq. 1 in log form, the quantity a prefill attention kernel keeps per query row.
    q_win [Hq, w, d], k [Hkv, S, d] -> [Hq, w] float64.
    """
    x = window_logits(q_win, k, scale)
    m = x.max(axis=-1)
    return m + np.log(np.exp(x - m[..., None]).sum(axis=-1))


def score_window_from_lse(q_win: np.ndarray, k: np.ndarray, lse: np.ndarray, P: int,
                          scale: Optional[float] = None, row_scale: float = 1.0) -> np.ndarray:
    """Steps O1-O5 with the softmax of Eq. 1 taken from supplied row normalisers: p = exp(x - lse[row]).

    With lse = row_lse(q_win, k) this is score_window; it lets the scoring run as ONE sweep over the keys when
    the caller (the prefill attention) already holds the normalisers of its last w query rows.
    lse [Hq, w] (natural log) -> A^l [Hkv, S'] float32.
    """
    Hq, w, _ = q_win.shape
    Hkv = k.shape[0]
    x = window_logits(q_win, k, scale)
    p = np.exp(x - np.asarray(lse, dtype=np.float64)[..., None])
    a = window_sum(p, Hkv, row_scale)
    return max_pool_prefix(a, w, P)


# --------------------------------------------------------------------------
# Eq. 3 / Algorithm 1 "indices <- A^l.topk(B^l, dim=-1).indices"
# --------------------------------------------------------------------------
def select_topk(A: np.ndarray, layer_max: int) -> np.ndarray:
    """O6: per KV head the k = min(B^l, S') best prefix positions, (score desc, index asc).

    A [Hkv, S'] float32 -> idx [Hkv, k] int32.
    """
    A = np.asarray(A, dtype=np.float32)
    Hkv, Sp = A.shape
    kk = min(layer_max, Sp)
    idx = np.empty((Hkv, kk), dtype=np.int32)
    for h in range(Hkv):
        order = np.argsort(-A[h].astype(np.float64), kind="stable")
        idx[h] = order[:kk]
    return idx


# --------------------------------------------------------------------------
# Algorithm 1 "K^b_l <- cat(K^s[:, :-ws].gather(indices), K^s[:, -ws:])"
# --------------------------------------------------------------------------
def gather_kv(k: np.ndarray, v: np.ndarray, idx: np.ndarray, w: int) -> Tuple[np.ndarray, np.ndarray]:
    """O7: buffer rows = selected prefix rows (in idx order) followed by the w window rows."""
    Hkv, S, d = k.shape
    n = idx.shape[1]
    kb = np.empty((Hkv, n + w, d), dtype=k.dtype)
    vb = np.empty((Hkv, n + w, d), dtype=v.dtype)
    for h in range(Hkv):
        kb[h, :n] = k[h, idx[h]]
        kb[h, n:] = k[h, S - w:]
        vb[h, :n] = v[h, idx[h]]
        vb[h, n:] = v[h, S - w:]
    return kb, vb


# --------------------------------------------------------------------------
# Decoding over the compressed cache (Section 4.3: the decoding phase is unchanged - ordinary attention of the
# new token over whatever keys and values the cache holds)
# --------------------------------------------------------------------------
def decode_attention(q_new: np.ndarray, kc: np.ndarray, vc: np.ndarray,
                     scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Attention of one new token over one layer's compressed cache.

    q_new [Hq, d]; kc, vc [Hkv, R, d] (R = retained + window rows, any order: the result does not depend on it).
    out[g] = sum_r softmax_r(scale * <q_new[g], kc[g // G, r]>) * vc[g // G, r]  -> [Hq, d] float64,
    lse[g] = log sum_r exp(scale * <q_new[g], kc[g // G, r]>)                    -> [Hq]    float64.
    """
    q = np.asarray(q_new, dtype=np.float64)
    k = np.asarray(kc, dtype=np.float64)
    v = np.asarray(vc, dtype=np.float64)
    Hq, d = q.shape
    Hkv, R, _ = k.shape
    assert Hq % Hkv == 0 and R >= 1
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((Hq, d), dtype=np.float64)
    lse = np.empty(Hq, dtype=np.float64)
    for g in range(Hq):
        x = scale * (k[g // G] @ q[g])
        m = x.max()
        e = np.exp(x - m)
        out[g] = (e / e.sum()) @ v[g // G]
        lse[g] = m + np.log(e.sum())
    return out, lse


# --------------------------------------------------------------------------
# Eq. 4-6 / Algorithm 1 "Update_Buffer_Length"
# --------------------------------------------------------------------------
def layer_hit_counts(A_list: Sequence[np.ndarray], mean_budget: int) -> np.ndarray:
    """Phi(TopK(A, (wt - ws) * H * l)) of Eq. 4: hits of the global top-k per layer.

    A_list: l arrays [Hkv, S'] float32 (layers processed so far).  The flat
    order is (layer, head, position); ties go to the lower flat index.
    """
    l = len(A_list)
    Hkv, Sp = A_list[0].shape
    flat = np.concatenate([np.asarray(a, dtype=np.float32).reshape(-1) for a in A_list])
    kg = min(mean_budget * Hkv * l, flat.size)
    order = np.argsort(-flat.astype(np.float64), kind="stable")[:kg]
    per_layer = Hkv * Sp
    cnt = np.zeros(l, dtype=np.int64)
    if per_layer > 0:
        np.add.at(cnt, order // per_layer, 1)
    return cnt


def budgets_from_counts(cnt: np.ndarray, layer_max: int, mean_budget: int, L: int) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 5-6: Z_i = floor(B^l * cnt_i / max cnt), Z'_i = floor(Z_i * B / sum Z), B = (wt - ws) * L.

    Exact integer arithmetic (python ints).  All-zero counts give all-zero budgets.
    """
    c = [int(x) for x in cnt]
    cmax = max(c) if c else 0
    if cmax == 0:
        z = [0] * len(c)
        return np.array(z, dtype=np.int64), np.array(z, dtype=np.int64)
    Z = [(layer_max * t) // cmax for t in c]
    total = sum(Z)
    B = mean_budget * L
    Zp = [(z * B) // total for z in Z]
    return np.array(Z, dtype=np.int64), np.array(Zp, dtype=np.int64)


def update_buffer_length(A_list: Sequence[np.ndarray], layer_max: int, mean_budget: int, L: int
                         ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """O8: (cnt, Z, Z') after the layers in A_list have been processed."""
    cnt = layer_hit_counts(A_list, mean_budget)
    Z, Zp = budgets_from_counts(cnt, layer_max, mean_budget, L)
    return cnt, Z, Zp


# --------------------------------------------------------------------------
# Fixed-pattern budget schedules: the comparison methods of Section 5.1 ("Baselines") and Figure 1 (b), (c),
# as alternative producers of the per-layer retained counts.  The paper names them in one sentence each and
# gives no formula, so each function states the reading it implements.
# --------------------------------------------------------------------------
def fixed_layer_budgets(L: int, mean_budget: int) -> np.ndarray:
    """Figure 1 (b): the same cache size in every layer, Z'_i = wt - ws.

    With Eq. 1-3 as the selection this is the SnapKV-style baseline: every layer keeps the top (wt - ws)
    prefix positions per KV head and no update ever runs.
    """
    return np.full(L, int(mean_budget), dtype=np.int64)


def pyramid_layer_budgets(L: int, mean_budget: int, layer_max: int, beta: int = 4) -> np.ndarray:
    """Figure 1 (c): retention that decreases monotonically with depth (the PyramidKV-style baseline).

    Reading: a straight line from `hi` rows at layer 0 to `lo` rows at layer L - 1 whose mean is the
    mean budget: lo = floor(mean_budget / beta), hi = 2 * mean_budget - lo, and if hi exceeds the
    per-layer maximum B^l it is lowered to B^l and lo raised by the same amount.  Layer i gets
    floor(((L - 1 - i) * hi + i * lo) / (L - 1)) (exact integers); L = 1 gets the mean budget.
    The sum is at most B = (wt - ws) * L and misses it by less than L.
    """
    assert L >= 1 and beta >= 1
    if L == 1:
        return np.array([int(mean_budget)], dtype=np.int64)
    lo = int(mean_budget) // int(beta)
    hi = 2 * int(mean_budget) - lo
    if hi > layer_max:
        lo += hi - int(layer_max)
        hi = int(layer_max)
    return np.array([((L - 1 - i) * hi + i * lo) // (L - 1) for i in range(L)], dtype=np.int64)


def recent_indices(prefix_len: int, budget: int, n_sink: int) -> np.ndarray:
    """StreamingLLM-style retention of one row of `prefix_len` candidate positions: the first n_sink positions
    (the attention sinks) and the most recent ones, budget positions in all (k = min(budget, prefix_len)).

    Order: the sinks in position order, then the recent positions from the newest to the oldest, so that
    keeping the first n entries of the list is again "sinks + the most recent" (the truncation rule of
    Algorithm 1 applies to this list unchanged).  No scores are involved; the window itself is always kept.
    """
    k = min(int(budget), int(prefix_len))
    sinks = min(int(n_sink), k)
    recent = k - sinks
    return np.concatenate([np.arange(sinks), prefix_len - 1 - np.arange(recent)]).astype(np.int32)


def apply_layer_budgets(n: Sequence[int], budgets: Sequence[int]) -> List[int]:
    """The truncation loop of Algorithm 1 with preset budgets: n_i <- min(n_i, budgets_i)."""
    return [min(int(a), int(b)) for a, b in zip(n, budgets)]


def compress_fixed_pattern(layers, L: int, w: int, P: int, layer_max: int, budgets: Sequence[int],
                           scale: Optional[float] = None, row_scale: float = 1.0, keep_buffers: bool = True,
                           scores_override: Optional[Sequence[np.ndarray]] = None,
                           n_sink: Optional[int] = None) -> "Compressed":
    """The layer loop of Algorithm 1 with a preset schedule instead of the progressive update: every layer is
    scored and selected as in Eq. 1-3 (k = min(B^l, S')), then truncated to budgets[l].  With n_sink given the
    candidates come from recent_indices (no scoring) instead of the top-k.
    """
    out = Compressed()
    for l, (q_win, k, v) in enumerate(layers, start=1):
        if n_sink is None:
            A = (np.asarray(scores_override[l - 1], dtype=np.float32) if scores_override is not None
                 else score_window(q_win, k, P, scale, row_scale))
            idx = select_topk(A, layer_max)
        else:
            Hkv, S = k.shape[0], k.shape[1]
            A = np.zeros((Hkv, S - w), dtype=np.float32)
            idx = np.tile(recent_indices(S - w, layer_max, n_sink), (Hkv, 1))
        out.A.append(A)
        out.idx.append(idx)
        out.n.append(idx.shape[1])
        if keep_buffers:
            kb, vb = gather_kv(k, v, idx, w)
            out.kb.append(kb)
            out.vb.append(vb)
    out.n = apply_layer_budgets(out.n, budgets)
    return out


# --------------------------------------------------------------------------
# Algorithm 1, the whole prefill loop for one sequence
# --------------------------------------------------------------------------
class Compressed:
    """Result of compress(): per-layer scores, ordered indices, counts and budgets."""

    def __init__(self):
        self.A: List[np.ndarray] = []          # A^b: pooled scores [Hkv, S'] float32 per layer
        self.idx: List[np.ndarray] = []        # ordered retained candidates [Hkv, k] per layer
        self.n: List[int] = []                 # retained prefix rows per head, per layer
        self.kb: List[np.ndarray] = []         # K^b_l  [Hkv, k + w, d]
        self.vb: List[np.ndarray] = []
        self.budgets: List[Tuple[int, np.ndarray, np.ndarray, np.ndarray]] = []  # (l, cnt, Z, Z')

    def cache(self, layer: int, w: int) -> Tuple[np.ndarray, np.ndarray]:
        """K^c_l, V^c_l: the first n_l buffer rows followed by the window rows."""
        n = self.n[layer]
        kb, vb = self.kb[layer], self.vb[layer]
        return (np.concatenate([kb[:, :n], kb[:, kb.shape[1] - w:]], axis=1),
                np.concatenate([vb[:, :n], vb[:, vb.shape[1] - w:]], axis=1))


def compress(layers, L: int, w: int, P: int, layer_max: int, mean_budget: int, interval: int,
             scale: Optional[float] = None, row_scale: float = 1.0, keep_buffers: bool = True,
             scores_override: Optional[Sequence[np.ndarray]] = None) -> Compressed:
    """Algorithm 1 for one sequence.

    layers: iterable yielding (q_win [Hq, w, d], k [Hkv, S, d], v [Hkv, S, d]) per layer.
    scores_override: if given, A^l is taken from it instead of being computed
    (used to check selection and budgets in isolation on a fixed float32 input).
    """
    out = Compressed()
    for l, (q_win, k, v) in enumerate(layers, start=1):
        A = (np.asarray(scores_override[l - 1], dtype=np.float32) if scores_override is not None
             else score_window(q_win, k, P, scale, row_scale))
        out.A.append(A)
        idx = select_topk(A, layer_max)
        out.idx.append(idx)
        out.n.append(idx.shape[1])
        if keep_buffers:
            kb, vb = gather_kv(k, v, idx, w)
            out.kb.append(kb)
            out.vb.append(vb)
        if l % interval == 0:
            cnt, Z, Zp = update_buffer_length(out.A, layer_max, mean_budget, L)
            out.budgets.append((l, cnt, Z, Zp))
            for i in range(l):
                out.n[i] = min(out.n[i], int(Zp[i]))
    return out
