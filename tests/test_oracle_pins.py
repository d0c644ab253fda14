"""Pins for the CPU oracle: closed forms, invariants, library special cases, brute force.

The paper prints no worked numeric example of Algorithm 1, so each oracle step
is pinned to something other than itself: the mathematics of Eq. 1-6, library
routines on the special cases that reduce to them, hand-worked budget rows
(tests/golden/budget_examples.txt) and pure-Python brute force on tiny inputs.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import dkv_oracle as O
from paper_2412_14838_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- O1-O4 (Eq. 1)
def test_unpooled_scores_sum_to_number_of_rows():
    """Every softmax row sums to 1 over all S keys => sum_s a[h, s] = G * w (Eq. 1)."""
    Hq, Hkv, w, d, S = 6, 2, 5, 16, 97
    q, k = _rand((Hq, w, d), 1), _rand((Hkv, S, d), 2)
    p = O.softmax_rows(O.window_logits(q, k))
    assert np.allclose(p.sum(axis=-1), 1.0, atol=1e-12)
    a = O.window_sum(p, Hkv)
    assert np.allclose(a.sum(axis=-1), (Hq // Hkv) * w, atol=1e-10)
    assert np.allclose(O.window_sum(p, Hkv, row_scale=1.0 / w).sum(axis=-1), Hq // Hkv, atol=1e-10)


def test_single_row_reduces_to_library_softmax():
    """w = 1, G = 1: the only window row sees all keys; score = softmax(q K^T / sqrt(d)) (Eq. 1)."""
    d, S = 32, 200
    q, k = _rand((1, 1, d), 3), _rand((1, S, d), 4)
    a = O.window_sum(O.softmax_rows(O.window_logits(q, k)), 1)
    ref = torch.softmax(torch.from_numpy(q[0]) @ torch.from_numpy(k[0]).T / math.sqrt(d), dim=-1).numpy()
    assert np.allclose(a[0], ref[0], rtol=1e-12, atol=1e-15)
    # P = 1 pooling is the identity on the prefix
    A = O.score_window(q, k, P=1)
    assert np.array_equal(A[0], ref[0, :S - 1].astype(np.float32))


def test_zero_queries_closed_form_proves_causal_mask():
    """Q = 0: window row i is uniform over its S - w + i + 1 visible keys, so every prefix
    score is G * sum_i 1 / (S - w + i + 1); without the causal mask it would be G * w / S."""
    Hq, Hkv, w, d, S = 4, 2, 8, 8, 50
    q, k = np.zeros((Hq, w, d)), _rand((Hkv, S, d), 5)
    a = O.window_sum(O.softmax_rows(O.window_logits(q, k)), Hkv)
    G = Hq // Hkv
    expect = G * sum(Fraction(1, S - w + i + 1) for i in range(w))
    assert np.allclose(a[:, :S - w], float(expect), rtol=1e-13)
    assert abs(float(expect) - G * w / S) > 1e-3
    # inside the window, column S - w + j is visible to rows i >= j only
    for j in range(w):
        col = G * sum(Fraction(1, S - w + i + 1) for i in range(j, w))
        assert np.allclose(a[:, S - w + j], float(col), rtol=1e-13)


def test_scale_is_one_over_sqrt_d_and_sign_is_right():
    """Hand example (Eq. 1): d = 4, one row q = (2,0,0,0), keys (1,..), (0,..), (-1,..):
    logits 2/2, 0, -2/2 => softmax = e^{1}, e^{0}, e^{-1} normalised."""
    q = np.array([[[2.0, 0, 0, 0]]])
    k = np.array([[[1.0, 0, 0, 0], [0, 0, 0, 0], [-1.0, 0, 0, 0]]])
    p = O.softmax_rows(O.window_logits(q, k))[0, 0]
    e = np.array([math.e, 1.0, 1.0 / math.e])
    assert np.allclose(p, e / e.sum(), rtol=1e-14)
    # explicit scale overrides the default
    p2 = O.softmax_rows(O.window_logits(q, k, scale=1.0))[0, 0]
    e2 = np.array([math.e ** 2, 1.0, math.e ** -2])
    assert np.allclose(p2, e2 / e2.sum(), rtol=1e-14)


def test_brute_force_scores_tiny():
    """Pure-Python loops over every (head, row, key) with math.exp, masked by position."""
    Hq, Hkv, w, d, S, P = 4, 2, 3, 5, 17, 3
    G = Hq // Hkv
    q, k = _rand((Hq, w, d), 6), _rand((Hkv, S, d), 7)
    a = [[0.0] * S for _ in range(Hkv)]
    for g in range(Hq):
        for i in range(w):
            last = S - w + i
            logits = [sum(q[g, i, t] * k[g // G, s, t] for t in range(d)) / math.sqrt(d) for s in range(last + 1)]
            mx = max(logits)
            den = sum(math.exp(x - mx) for x in logits)
            for s in range(last + 1):
                a[g // G][s] += math.exp(logits[s] - mx) / den
    Sp = S - w
    pooled = [[max(a[h][max(0, s - 1):min(Sp - 1, s + 1) + 1]) for s in range(Sp)] for h in range(Hkv)]
    A = O.score_window(q, k, P)
    assert A.dtype == np.float32 and A.shape == (Hkv, Sp)
    assert np.allclose(A, np.array(pooled), rtol=1e-6)


def test_gqa_is_the_sum_of_its_query_heads():
    """Linearity of the group reduction: G = 4 scores = sum of four G = 1 runs on the same K."""
    G, w, d, S = 4, 4, 16, 64
    q, k = _rand((G, w, d), 8), _rand((1, S, d), 9)
    full = O.window_sum(O.softmax_rows(O.window_logits(q, k)), 1)
    parts = sum(O.window_sum(O.softmax_rows(O.window_logits(q[g:g + 1], k)), 1) for g in range(G))
    assert np.allclose(full, parts, rtol=1e-13)
    # heads of different KV groups do not mix
    k2 = _rand((2, S, d), 10)
    both = O.window_sum(O.softmax_rows(O.window_logits(q, k2)), 2)
    only0 = O.window_sum(O.softmax_rows(O.window_logits(q[:2], k2[:1])), 1)
    assert np.allclose(both[0], only0[0], rtol=1e-13)


# ---------------------------------------------------------------- O5 (Eq. 2)
def test_pool_matches_library_max_pool_on_prefix():
    Hkv, S, w = 3, 101, 9
    a = np.abs(_rand((Hkv, S), 11))
    for P in (1, 3, 7, 13):
        got = O.max_pool_prefix(a, w, P)
        pre = torch.from_numpy(a[:, :S - w]).unsqueeze(0)
        ref = torch.nn.functional.max_pool1d(pre, kernel_size=P, stride=1, padding=(P - 1) // 2)[0].numpy()
        assert np.array_equal(got, ref.astype(np.float32))


def test_pool_spike_and_window_isolation():
    """A single spike spreads to exactly P positions (clipped at the ends); a large value in
    the first window column must not leak into the last prefix positions."""
    S, w, P = 40, 8, 7
    Sp = S - w
    for spike in (0, 2, 15, Sp - 1):
        a = np.zeros((1, S))
        a[0, spike] = 5.0
        a[0, Sp] = 99.0              # first window column
        A = O.max_pool_prefix(a, w, P)[0]
        lo, hi = max(0, spike - 3), min(Sp - 1, spike + 3)
        expect = np.zeros(Sp, dtype=np.float32)
        expect[lo:hi + 1] = 5.0
        assert np.array_equal(A, expect)


# ---------------------------------------------------------------- O6 (Eq. 3)
def test_select_brute_force_and_ties():
    rng = np.random.default_rng(12)
    for trial in range(20):
        Sp = int(rng.integers(1, 60))
        # few distinct values => many exact ties
        A = rng.integers(0, 5, size=(2, Sp)).astype(np.float32) / 4
        kmax = int(rng.integers(1, 70))
        got = O.select_topk(A, kmax)
        for h in range(2):
            brute = sorted(range(Sp), key=lambda s: (-float(A[h, s]), s))[:min(kmax, Sp)]
            assert got[h].tolist() == brute
    assert O.select_topk(np.ones((1, 10), dtype=np.float32), 4)[0].tolist() == [0, 1, 2, 3]
    # the selected values agree with the library's top-k values
    A = np.abs(_rand((3, 500), 13)).astype(np.float32)
    got = O.select_topk(A, 37)
    ref = torch.topk(torch.from_numpy(A), 37, dim=-1).values.numpy()
    assert np.array_equal(np.take_along_axis(A, got, axis=1), ref)


# ---------------------------------------------------------------- O7
def test_gather_rows_are_copies():
    Hkv, S, d, w = 2, 30, 4, 5
    k, v = _rand((Hkv, S, d), 14).astype(np.float32), _rand((Hkv, S, d), 15).astype(np.float32)
    idx = np.array([[7, 0, 24, 3], [1, 2, 23, 11]], dtype=np.int32)
    kb, vb = O.gather_kv(k, v, idx, w)
    assert kb.shape == (Hkv, 4 + w, d)
    for h in range(Hkv):
        for j, s in enumerate(idx[h]):
            assert np.array_equal(kb[h, j], k[h, s]) and np.array_equal(vb[h, j], v[h, s])
        assert np.array_equal(kb[h, 4:], k[h, S - w:]) and np.array_equal(vb[h, 4:], v[h, S - w:])


# ---------------------------------------------------------------- O8 (Eq. 4-6)
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "budget_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [[int(x) for x in p.split()] for p in line.split("|")]
            rows.append(parts)
    return rows


def test_budget_formulas_against_hand_worked_rows():
    rows = _golden_rows()
    assert len(rows) >= 6
    for (layer_max, mean_budget, L), cnt, Z, Zp in rows:
        gotZ, gotZp = O.budgets_from_counts(np.array(cnt), layer_max, mean_budget, L)
        assert gotZ.tolist() == Z and gotZp.tolist() == Zp


def test_budget_normalisation_cancels_in_exact_arithmetic():
    """The listing divides the counts by l and normalises them to (0, 1) before t / max(norm);
    in exact rational arithmetic any positive rescaling cancels (Eq. 5), and r = sum(Z)/B."""
    rng = np.random.default_rng(16)
    for _ in range(50):
        l = int(rng.integers(1, 9))
        L = l + int(rng.integers(0, 4))
        cnt = rng.integers(0, 5000, size=l)
        cnt[int(rng.integers(0, l))] += 1
        layer_max, mean_budget = int(rng.integers(1, 3000)), int(rng.integers(1, 700))
        norm = [Fraction(int(c), l) / Fraction(int(cnt.sum()), l) for c in cnt]
        Z = [math.floor(layer_max * t / max(norm)) for t in norm]
        r = Fraction(sum(Z), mean_budget * L)
        Zp = [math.floor(z / r) for z in Z]
        gotZ, gotZp = O.budgets_from_counts(cnt, layer_max, mean_budget, L)
        assert gotZ.tolist() == Z and gotZp.tolist() == Zp
        B = mean_budget * L
        assert B - l < sum(Zp) <= B
    z, zp = O.budgets_from_counts(np.zeros(3, dtype=np.int64), 10, 5, 3)
    assert z.tolist() == [0, 0, 0] and zp.tolist() == [0, 0, 0]


def test_layer_hit_counts_brute_force_and_ties():
    rng = np.random.default_rng(17)
    for _ in range(10):
        l, Hkv, Sp = int(rng.integers(1, 5)), 2, int(rng.integers(3, 40))
        A_list = [(rng.integers(0, 6, size=(Hkv, Sp)) / 5).astype(np.float32) for _ in range(l)]
        mean_budget = int(rng.integers(1, Sp + 5))
        cnt = O.layer_hit_counts(A_list, mean_budget)
        flat = [(-float(A_list[i][h, s]), (i * Hkv + h) * Sp + s) for i in range(l) for h in range(Hkv) for s in range(Sp)]
        kg = min(mean_budget * Hkv * l, len(flat))
        brute = [0] * l
        for _, fi in sorted(flat)[:kg]:
            brute[fi // (Hkv * Sp)] += 1
        assert cnt.tolist() == brute and int(cnt.sum()) == kg
    # bit-equal scores everywhere: the earlier layers win the ties
    same = [np.ones((2, 10), dtype=np.float32) for _ in range(3)]
    assert O.layer_hit_counts(same, 4).tolist() == [20, 4, 0]
    # all mass in one layer
    A_list = [np.zeros((2, 10), dtype=np.float32), np.ones((2, 10), dtype=np.float32)]
    assert O.layer_hit_counts(A_list, 5).tolist() == [0, 20]


def test_flat_counts_give_the_fixed_budget_pattern():
    """Equal hit counts => Z' = floor(mean_budget * L / l); at l = L that is the fixed per-layer budget."""
    for l, L in ((4, 4), (2, 4), (8, 32)):
        _, Zp = O.budgets_from_counts(np.full(l, 77), 512, 128, L)
        assert Zp.tolist() == [(512 * 128 * L) // (512 * l)] * l


# ---------------------------------------------------------------- Algorithm 1 as a whole
def _layers(cfg, seq=0):
    cu = cfg.cu_seqlens
    for l in range(cfg.L):
        d = W.make_layer(cfg, l)
        yield d["q_win"][seq], d["k"][:, cu[seq]:cu[seq + 1]], d["v"][:, cu[seq]:cu[seq + 1]]


@pytest.mark.parametrize("normalize", [False, True])
def test_driver_invariants_on_tiny(normalize):
    cfg = W.standard_configs()["tiny"].with_(plant_normalize=normalize)
    S, w = cfg.seqlens[0], cfg.w
    r = O.compress(_layers(cfg), cfg.L, w, cfg.P, cfg.layer_max, cfg.mean_budget, cfg.interval)
    B = cfg.global_budget
    prev = [cfg.layer_max] * cfg.L
    for (l, cnt, Z, Zp) in r.budgets:
        assert l % cfg.interval == 0 and len(cnt) == l
        assert int(cnt.sum()) == min(cfg.mean_budget * cfg.Hkv * l, l * cfg.Hkv * (S - w))
        assert int(Z.max()) == cfg.layer_max and B - l < int(Zp.sum()) <= B
    for i in range(cfg.L):
        assert 0 <= r.n[i] <= cfg.layer_max and r.n[i] <= prev[i]
        assert r.n[i] == min(cfg.layer_max, int(r.budgets[-1][3][i]), *(int(b[3][i]) for b in r.budgets if b[0] > i))
        kc, vc = r.cache(i, w)
        assert kc.shape == (cfg.Hkv, r.n[i] + w, cfg.d)
        assert sum(r.n) <= B
    if normalize:
        # calibrated planting: every planted key is among the layer's candidates, ranked first, all tied
        for l in range(cfg.L):
            pos = W.planted_positions(cfg, l, 0)
            for h in range(cfg.Hkv):
                # pooling spreads every planted spike over P tied neighbours
                top = r.idx[l][h][:cfg.P * len(pos)]
                assert len(np.unique(r.A[l][h][pos])) == 1
                if cfg.P * len(pos) <= r.idx[l].shape[1]:
                    assert np.isin(pos, top).all()
                else:   # more tied plateau positions than candidates: all candidates carry the planted score
                    assert (r.A[l][h][r.idx[l][h]] == r.A[l][h][pos[0]]).all()


def test_scores_override_isolates_selection():
    cfg = W.standard_configs()["tiny"]
    r = O.compress(_layers(cfg), cfg.L, cfg.w, cfg.P, cfg.layer_max, cfg.mean_budget, cfg.interval)
    r2 = O.compress(_layers(cfg), cfg.L, cfg.w, cfg.P, cfg.layer_max, cfg.mean_budget, cfg.interval,
                    scores_override=r.A, keep_buffers=False)
    assert r.n == r2.n and all(np.array_equal(a, b) for a, b in zip(r.idx, r2.idx))


def _hand_case_for_the_final_cache():
    """Two layers, two KV heads, S = 10, ws = 2 (prefix 8), B^l = 4, mean budget 3, one update after layer 2.
    Key row (layer l, head h, position s) = [100 l + 10 h + s, -(100 l + 10 h + s)], value = key + 0.5, so every
    cache row names where it came from.  Scores are supplied, so that everything below follows by hand."""
    L, Hkv, S, w, d = 2, 2, 10, 2, 2
    layers = []
    for l in range(L):
        base = (100 * l + 10 * np.arange(Hkv)[:, None] + np.arange(S)[None, :]).astype(np.float64)
        k = np.stack([base, -base], axis=-1)
        layers.append((None, k, k + 0.5))
    A = [np.array([[.90, .10, .80, .20, .70, .30, .60, .05],      # layer 1 head 0: order 0, 2, 4, 6
                   [.15, .95, .25, .85, .35, .75, .45, .65]],     #         head 1: order 1, 3, 5, 7
                  dtype=np.float32),
         np.array([[.01, .91, .02, .81, .03, .04, .05, .06],      # layer 2 head 0: order 1, 3, 7, 6
                   [.71, .07, .61, .08, .09, .11, .12, .13]],     #         head 1: order 0, 2, 7, 6
                  dtype=np.float32)]
    return layers, A, dict(L=L, w=w, P=1, layer_max=4, mean_budget=3, interval=2)


def test_final_cache_rows_of_a_hand_worked_case():
    """Algorithm 1, last line, after the truncation lines: K^c_l = the first n_l buffer rows, then the ws window
    rows.  By hand: kg = 3 * 2 * 2 = 12; the 12 largest of the 32 scores are .95 .91 .90 .85 .81 .80 .75 .71 .70
    .65 .61 .60, eight of them in layer 1 and four in layer 2: cnt = [8, 4]; Z = [4 * 8 / 8, 4 * 4 / 8] = [4, 2];
    sum Z = 6 = B, so Z' = [4, 2] and n = [4, 2]: layer 2 keeps only the first TWO of its four selected rows."""
    layers, A, kw = _hand_case_for_the_final_cache()
    r = O.compress(layers, scores_override=A, **kw)
    assert r.budgets[0][1].tolist() == [8, 4] and r.budgets[0][3].tolist() == [4, 2] and r.n == [4, 2]
    assert r.idx[1].tolist() == [[1, 3, 7, 6], [0, 2, 7, 6]]
    kc0, vc0 = r.cache(0, kw["w"])
    kc1, vc1 = r.cache(1, kw["w"])
    # layer 1 (index 0): all four selected rows of each head, then the window rows 8 and 9
    assert kc0[:, :, 0].tolist() == [[0, 2, 4, 6, 8, 9], [11, 13, 15, 17, 18, 19]]
    # layer 2 (index 1): rows 1, 3 (head 0) and 0, 2 (head 1) survive the update, then the window rows
    assert kc1[:, :, 0].tolist() == [[101, 103, 108, 109], [110, 112, 118, 119]]
    for kc, vc in ((kc0, vc0), (kc1, vc1)):
        assert np.array_equal(kc[:, :, 1], -kc[:, :, 0]) and np.array_equal(vc, kc + 0.5)


# ---------------------------------------------------------------- fixed-pattern schedules (Section 5.1, Figure 1)
def _schedule_rows(kind):
    with open(os.path.join(GOLDEN, "schedule_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if line.startswith(kind + " "):
                left, right = line[len(kind):].split("|")
                yield [int(x) for x in left.split()], [int(x) for x in right.split()]


def test_schedules_against_hand_worked_rows():
    rows = list(_schedule_rows("pyramid"))
    assert len(rows) >= 5
    for (L, mean, layer_max, beta), want in rows:
        assert O.pyramid_layer_budgets(L, mean, layer_max, beta).tolist() == want
    for (L, mean), want in _schedule_rows("fixed"):
        assert O.fixed_layer_budgets(L, mean).tolist() == want
    rows = list(_schedule_rows("recent"))
    assert len(rows) >= 5
    for (prefix, budget, n_sink), want in rows:
        assert O.recent_indices(prefix, budget, n_sink).tolist() == want


def test_pyramid_schedule_invariants():
    """Monotone non-increasing, first layer hi and last layer lo exactly, every layer within B^l, and the sum
    within L of the global budget B = mean * L from below (the straight line has mean exactly `mean`)."""
    for L, mean, layer_max, beta in ((32, 512, 2048, 4), (28, 64, 256, 4), (32, 128, 150, 8), (5, 7, 9, 3), (2, 1, 1, 2)):
        z = O.pyramid_layer_budgets(L, mean, layer_max, beta)
        lo = mean // beta
        hi = 2 * mean - lo
        if hi > layer_max:
            lo, hi = lo + hi - layer_max, layer_max
        assert (np.diff(z) <= 0).all() and z[0] == hi and z[-1] == lo and z.max() <= layer_max and z.min() >= 0
        assert mean * L - L < z.sum() <= mean * L
        # the exact line, in rationals
        assert z.tolist() == [int(Fraction((L - 1 - i) * hi + i * lo, L - 1)) for i in range(L)]


def test_fixed_pattern_loop_is_per_layer_topk_cut_to_the_schedule():
    """With the fixed schedule the loop is Eq. 1-3 with k = the mean budget in every layer (brute-force sort);
    with any schedule n_l = min(B^l, S', budgets_l) and the retained list is a prefix of the B^l list."""
    cfg = W.standard_configs()["tiny"]
    S, w = cfg.seqlens[0], cfg.w
    fixed = O.fixed_layer_budgets(cfg.L, cfg.mean_budget)
    r = O.compress_fixed_pattern(_layers(cfg), cfg.L, w, cfg.P, cfg.layer_max, fixed)
    assert r.n == [cfg.mean_budget] * cfg.L and r.budgets == []
    for l, (q, k, v) in enumerate(_layers(cfg)):
        A = O.score_window(q, k, cfg.P)
        for h in range(cfg.Hkv):
            brute = sorted(range(S - w), key=lambda s: (-float(A[h, s]), s))[:cfg.mean_budget]
            assert r.idx[l][h][:r.n[l]].tolist() == brute
        kc, vc = r.cache(l, w)
        assert kc.shape[1] == cfg.mean_budget + w and np.array_equal(kc[:, -w:], k[:, S - w:])
    pyr = O.pyramid_layer_budgets(cfg.L, cfg.mean_budget, cfg.layer_max, 4)
    r2 = O.compress_fixed_pattern(_layers(cfg), cfg.L, w, cfg.P, cfg.layer_max, pyr)
    assert r2.n == [min(cfg.layer_max, S - w, int(b)) for b in pyr]
    assert all(np.array_equal(a, b) for a, b in zip(r.idx, r2.idx))
    # the recency pattern: no scores, sinks + newest prefix rows, the window rows behind them
    r3 = O.compress_fixed_pattern(_layers(cfg), cfg.L, w, cfg.P, cfg.layer_max, fixed, n_sink=4)
    kc, _ = r3.cache(0, w)
    k0 = next(iter(_layers(cfg)))[1]
    want = list(range(4)) + list(range(S - w - 1, S - w - 1 - (cfg.mean_budget - 4), -1)) + list(range(S - w, S))
    assert np.array_equal(kc, k0[:, want])


# ---------------------------------------------------------------- Eq. 1 with supplied row normalisers
def test_row_lse_matches_library_logsumexp_and_closed_form():
    """lse[g, i] = log of the denominator of Eq. 1 over the keys the row may see: torch.logsumexp on the masked
    logits computed independently here, and the closed form log(S - w + i + 1) for zero queries."""
    Hq, Hkv, w, d, S = 4, 2, 3, 8, 41
    q, k = _rand((Hq, w, d), 31), _rand((Hkv, S, d), 32)
    lse = O.row_lse(q, k)
    G = Hq // Hkv
    for g in range(Hq):
        for i in range(w):
            visible = S - w + i + 1
            x = torch.tensor((q[g, i] @ k[g // G, :visible].T) / math.sqrt(d))
            assert abs(lse[g, i] - torch.logsumexp(x, dim=0).item()) < 1e-12
    zero = O.row_lse(np.zeros((Hq, w, d)), k)
    assert np.allclose(zero, np.log(S - w + np.arange(w) + 1.0)[None, :], atol=1e-13)


def test_scores_from_supplied_lse():
    """With the true normalisers the single-sweep form equals the softmax form; shifting a row's lse by delta
    scales that row's contribution by exp(-delta) (so a wrong sign or a missing row shows)."""
    Hq, Hkv, w, d, S, P = 4, 2, 4, 16, 120, 5
    q, k = _rand((Hq, w, d), 33), _rand((Hkv, S, d), 34)
    lse = O.row_lse(q, k)
    want = O.score_window(q, k, P)
    got = O.score_window_from_lse(q, k, lse, P)
    assert np.allclose(got, want, rtol=1e-6, atol=0)
    # unpooled: a[h, s] = sum_rows exp(x - lse); shift all rows of KV head 0 by log 2, of head 1 by -log 3
    shift = np.zeros((Hq, w))
    shift[:2] = math.log(2.0)
    shift[2:] = -math.log(3.0)
    base = O.score_window_from_lse(q, k, lse, 1)
    moved = O.score_window_from_lse(q, k, lse + shift, 1)
    assert np.allclose(moved[0], base[0] / 2.0, rtol=1e-6) and np.allclose(moved[1], base[1] * 3.0, rtol=1e-6)
    # brute force of one position
    h, s = 1, 17
    acc = 0.0
    for g in (2, 3):
        for i in range(w):
            acc += math.exp(float(q[g, i] @ k[h, s]) / math.sqrt(d) - lse[g, i])
    assert abs(base[h, s] - np.float32(acc)) <= 1e-6 * acc


# ---------------------------------------------------------------- decoding over the compressed cache
def test_decode_attention_against_library_and_special_cases():
    """Ordinary softmax attention of one query per head (Section 4.3): equals torch's scaled_dot_product_attention
    with the KV heads repeated G times; does not depend on the order of the cached rows; one row returns that row
    of V; a zero query returns the mean of V and lse = log R."""
    Hq, Hkv, d, R = 6, 2, 16, 37
    G = Hq // Hkv
    q, k, v = _rand((Hq, d), 41), _rand((Hkv, R, d), 42), _rand((Hkv, R, d), 43)
    out, lse = O.decode_attention(q, k, v)
    tq = torch.tensor(q)[:, None, :]                                 # [Hq, 1, d]
    tk = torch.tensor(np.repeat(k, G, axis=0))                       # [Hq, R, d]
    tv = torch.tensor(np.repeat(v, G, axis=0))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, 0, :].numpy()
    assert np.allclose(out, ref, rtol=1e-10, atol=1e-12)
    x = torch.einsum("gd,grd->gr", torch.tensor(q), tk) / math.sqrt(d)
    assert np.allclose(lse, torch.logsumexp(x, dim=1).numpy(), atol=1e-12)
    perm = np.random.default_rng(5).permutation(R)
    out_p, lse_p = O.decode_attention(q, k[:, perm], v[:, perm])
    assert np.allclose(out_p, out, atol=1e-12) and np.allclose(lse_p, lse, atol=1e-12)
    one, _ = O.decode_attention(q, k[:, 3:4], v[:, 3:4])
    assert np.allclose(one, np.repeat(v[:, 3], G, axis=0), atol=1e-13)
    zero, lse0 = O.decode_attention(np.zeros((Hq, d)), k, v)
    assert np.allclose(zero, np.repeat(v.mean(axis=1), G, axis=0), atol=1e-12) and np.allclose(lse0, math.log(R))
    # the scale: doubling q equals doubling the scale
    a, _ = O.decode_attention(2 * q, k, v)
    b, _ = O.decode_attention(q, k, v, scale=2.0 / math.sqrt(d))
    assert np.allclose(a, b, atol=1e-12)


# ---------------------------------------------------------------- planted mistakes must be caught
def test_pins_catch_planted_mistakes(monkeypatch):
    """Plant plausible mistakes in the oracle (on the CPU) and check that a pin fails."""
    def fails(fn):
        try:
            fn()
        except AssertionError:
            return True
        return False

    orig_logits = O.window_logits

    def no_mask(q, k, scale=None):
        q64, k64 = np.asarray(q, np.float64), np.asarray(k, np.float64)
        G = q64.shape[0] // k64.shape[0]
        sc = 1.0 / np.sqrt(q64.shape[-1]) if scale is None else scale
        return np.stack([sc * (q64[g] @ k64[g // G].T) for g in range(q64.shape[0])])

    monkeypatch.setattr(O, "window_logits", no_mask)
    assert fails(test_zero_queries_closed_form_proves_causal_mask)
    assert fails(test_brute_force_scores_tiny)
    monkeypatch.setattr(O, "window_logits", lambda q, k, scale=None: orig_logits(q, k, 1.0 if scale is None else scale))
    assert fails(test_scale_is_one_over_sqrt_d_and_sign_is_right)
    monkeypatch.setattr(O, "window_logits", lambda q, k, scale=None: -orig_logits(q, k, scale))
    assert fails(test_brute_force_scores_tiny)
    monkeypatch.setattr(O, "window_logits", orig_logits)

    orig_lse = O.row_lse
    monkeypatch.setattr(O, "row_lse", lambda q, k, scale=None: orig_logits(q, k, scale).max(axis=-1))   # max, not lse
    assert fails(test_row_lse_matches_library_logsumexp_and_closed_form)
    assert fails(test_scores_from_supplied_lse)
    monkeypatch.setattr(O, "row_lse", orig_lse)
    orig_from = O.score_window_from_lse
    monkeypatch.setattr(O, "score_window_from_lse",
                        lambda q, k, lse, P, scale=None, row_scale=1.0: orig_from(q, k, -np.asarray(lse), P, scale, row_scale))
    assert fails(test_scores_from_supplied_lse)
    monkeypatch.setattr(O, "score_window_from_lse", orig_from)

    orig_dec = O.decode_attention

    def wrong_head(q, k, v, scale=None):      # KV head by g % Hkv instead of g // G
        Hq, Hkv = np.asarray(q).shape[0], np.asarray(k).shape[0]
        order = [g % Hkv for g in range(Hq)]
        return orig_dec(q, np.asarray(k)[order], np.asarray(v)[order], scale)

    monkeypatch.setattr(O, "decode_attention", wrong_head)
    assert fails(test_decode_attention_against_library_and_special_cases)
    monkeypatch.setattr(O, "decode_attention", lambda q, k, v, scale=None: orig_dec(q, k, v, 1.0 if scale is None else scale))
    assert fails(test_decode_attention_against_library_and_special_cases)
    monkeypatch.setattr(O, "decode_attention", orig_dec)

    orig_pool = O.max_pool_prefix
    monkeypatch.setattr(O, "max_pool_prefix", lambda a, w, P: orig_pool(a, 0, P)[:, :a.shape[1] - w])
    assert fails(test_pool_spike_and_window_isolation)
    monkeypatch.setattr(O, "max_pool_prefix", orig_pool)

    orig_sel = O.select_topk
    monkeypatch.setattr(O, "select_topk", lambda A, m: np.stack(
        [np.argsort(-A[h], kind="stable")[::-1][:min(m, A.shape[1])][::-1] for h in range(A.shape[0])]).astype(np.int32))
    assert fails(test_select_brute_force_and_ties)
    monkeypatch.setattr(O, "select_topk", orig_sel)

    orig_b = O.budgets_from_counts

    def rounded(cnt, layer_max, mean_budget, L):
        c = np.asarray(cnt, dtype=np.float64)
        Z = np.round(layer_max * c / c.max())
        return Z.astype(np.int64), np.round(Z * mean_budget * L / Z.sum()).astype(np.int64)

    monkeypatch.setattr(O, "budgets_from_counts", rounded)
    assert fails(test_budget_formulas_against_hand_worked_rows)
    monkeypatch.setattr(O, "budgets_from_counts", orig_b)

    orig_cache = O.Compressed.cache

    def window_from_the_wrong_end(self, layer, w):      # the first w buffer rows instead of the last w
        n = self.n[layer]
        kb, vb = self.kb[layer], self.vb[layer]
        return np.concatenate([kb[:, :n], kb[:, :w]], axis=1), np.concatenate([vb[:, :n], vb[:, :w]], axis=1)

    monkeypatch.setattr(O.Compressed, "cache", window_from_the_wrong_end)
    assert fails(test_final_cache_rows_of_a_hand_worked_case)
    monkeypatch.setattr(O.Compressed, "cache", lambda self, layer, w: tuple(
        np.concatenate([b[:, :b.shape[1] - w], b[:, b.shape[1] - w:]], axis=1) for b in (self.kb[layer], self.vb[layer])))
    assert fails(test_final_cache_rows_of_a_hand_worked_case)       # no truncation to n_l
    monkeypatch.setattr(O.Compressed, "cache", orig_cache)

    orig_pyr = O.pyramid_layer_budgets
    monkeypatch.setattr(O, "pyramid_layer_budgets", lambda L, m, lm, beta=4: orig_pyr(L, m, lm, beta)[::-1].copy())
    assert fails(test_schedules_against_hand_worked_rows) and fails(test_pyramid_schedule_invariants)
    monkeypatch.setattr(O, "pyramid_layer_budgets", lambda L, m, lm, beta=4: np.minimum(orig_pyr(L, m, 10**9, beta), lm))
    assert fails(test_schedules_against_hand_worked_rows)           # a cap without moving the excess to lo
    monkeypatch.setattr(O, "pyramid_layer_budgets", orig_pyr)
    orig_recent = O.recent_indices
    monkeypatch.setattr(O, "recent_indices", lambda p, b, s: np.sort(orig_recent(p, b, s)))
    assert fails(test_schedules_against_hand_worked_rows)           # position order instead of newest first
    monkeypatch.setattr(O, "recent_indices", orig_recent)
