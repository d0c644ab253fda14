"""Host logic of the layer loop (CPU): which stage calls the two schedules issue, in which order.

The stage calls themselves are replaced by recorders; the buffers live on the CPU. What is checked is what the
results rest on: every layer is scored, selected and compacted exactly once, a layer is selected after it is
scored and compacted after it is selected, every update boundary is updated exactly once, in order, after the
selection of all layers below it, and the grouped schedule compacts a layer only after the updates of its group.
"""
import pytest
import torch

from paper_2412_14838_amd import dkv, workloads as W
from paper_2412_14838_amd import pipeline as P


def _record(monkeypatch):
    calls = []

    def rec(name, layers_of):
        def f(*args, **kw):
            calls.append((name, layers_of(*args)))
        return f

    monkeypatch.setattr(dkv, "dkv_score_window", rec("score", lambda desc, q, k, st, sh, cu, out, *a: None))
    monkeypatch.setattr(dkv, "dkv_score_window_layers",
                        rec("score", lambda desc, l0, qs, ks, *a: list(range(l0, l0 + len(ks)))))
    monkeypatch.setattr(dkv, "dkv_select_topk", rec("select", lambda desc, l, *a: [l]))
    monkeypatch.setattr(dkv, "dkv_select_topk_layers", rec("select", lambda desc, l0, n, *a: list(range(l0, l0 + n))))
    monkeypatch.setattr(dkv, "dkv_gather_kv", rec("gather", lambda desc, l, *a: [l]))
    monkeypatch.setattr(dkv, "dkv_gather_kv_layers",
                        rec("gather", lambda desc, l0, ks, *a: list(range(l0, l0 + len(ks)))))
    monkeypatch.setattr(dkv, "dkv_rebalance", rec("update", lambda desc, l, *a: [l]))
    monkeypatch.setattr(dkv, "dkv_rebalance_batch",
                        rec("update", lambda desc, l, n, *a: [l + u * desc.interval for u in range(n)]))
    return calls


@pytest.mark.parametrize("L,interval,group", [(8, 2, 1), (8, 2, 8), (8, 2, 3), (8, 4, 8), (7, 2, 4), (6, 1, 8), (5, 5, 2),
                                              (16, 2, 8), (32, 4, 32), (32, 2, 32), (40, 4, 64), (28, 4, 28)])
def test_schedules_issue_every_stage_once_and_in_a_valid_order(monkeypatch, L, interval, group):
    cfg = W.Workload("sched", L=L, Hq=4, Hkv=2, d=64, seqlens=(300, 70), dtype="f32", w=16, P=7, mean_budget=32,
                     layer_max=64, interval=interval, seed=1)
    calls = _record(monkeypatch)
    comp = P.Compressor(cfg, device="cpu", group=group)
    seen = []
    comp.on_update = seen.append
    dummy = torch.zeros(1)
    for l in range(L):
        # the single-layer score call does not say which layer it is for: note it here
        before = len(calls)
        comp.step(l, dummy, dummy, dummy)
        for i in range(before, len(calls)):
            if calls[i] == ("score", None):
                calls[i] = ("score", [l])
    when = {}
    for t, (name, layers) in enumerate(calls):
        for l in layers:
            assert (name, l) not in when, (name, l)          # exactly once
            when[(name, l)] = t
    boundaries = [b for b in range(interval, L + 1, interval)]
    for l in range(L):
        assert when[("score", l)] < when[("select", l)] < when[("gather", l)]
    assert [l for name, ls in calls if name == "update" for l in ls] == boundaries     # once each, in order
    assert seen == boundaries
    for b in boundaries:
        assert all(when[("select", l)] < when[("update", b)] for l in range(b))
    if group > 1:
        for l in range(L):        # compaction after the updates that the layer's group contains
            g0 = l // comp.group * comp.group
            inside = [b for b in boundaries if g0 < b <= min(g0 + comp.group, L)]
            assert all(when[("update", b)] < when[("gather", l)] for b in inside)
    # no call covers more than the library takes at once
    assert all(len(ls) <= dkv.DKV_MAX_SELECT_LAYERS for name, ls in calls if name != "update")
    assert all(len(ls) <= dkv.DKV_MAX_UPDATES for name, ls in calls if name == "update")
