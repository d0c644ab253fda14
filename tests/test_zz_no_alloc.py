"""The entry point that allocates nothing (dkv_score_window_static) against dkv_score_window, through the C ABI:
two calls in a row, the second with a smaller input, must each give bit-identical scores. The first call on a
device resolves the address of the library's fixed array (the runtime loads the code object that holds it then);
from the second call on the device's free memory must not shrink during a call."""
import gc

import numpy as np
import pytest
import torch

from oracle import dkv_oracle as O
from paper_2412_14838_amd import workloads as W
from paper_2412_14838_amd.pipeline import Compressor, to_device

pytestmark = pytest.mark.gpu


def _cfg(name, **kw):
    base = dict(name=name, L=2, Hq=8, Hkv=2, d=128, seqlens=(3000, 700), dtype="bf16", w=32, P=7, mean_budget=64,
                layer_max=160, interval=2, seed=91, plant="loguniform", plant_lo=4, plant_hi=40, gain=3.0,
                plant_normalize=True)
    base.update(kw)
    return W.Workload(**base)


@pytest.mark.parametrize("kind", ["bf16_mfma", "f32_valu"])
def test_static_scratch_scoring_equals_workspace_scoring(dkv, kind):
    big = _cfg("static_big") if kind == "bf16_mfma" else _cfg("static_big_f32", dtype="f32", d=64, w=16, seqlens=(2100, 300))
    small = big.with_(name="static_small", seqlens=(900,), seed=92)
    for cfg in (big, small):                     # two calls in a row, the second with a smaller input
        data = W.make_layer(cfg, 0, with_v=False)
        dev = to_device(cfg, data)
        comp = Compressor(cfg, keep_cache=False)
        T, d = cfg.total_tokens, cfg.d
        comp.score(0, dev["q_win"], dev["k"])                                   # the existing entry point
        out = torch.full_like(comp.scores[1], 7.0)
        gc.collect()                        # tensors of earlier tests must not be freed in the middle of the comparison
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]        # hipMemGetInfo: sees every allocation, not only torch's
        dkv.dkv_score_window_static(comp.desc, dev["q_win"], dev["k"], d, T * d, comp.cu, out, T)
        torch.cuda.synchronize()
        assert cfg is big or torch.cuda.mem_get_info()[0] >= free_before
        assert torch.equal(out.view(torch.int32), comp.scores[0].view(torch.int32)), cfg.name
        # and against the oracle, to the bar of the scoring tests
        cu = cfg.cu_seqlens
        got = out.cpu().numpy()
        for s in range(cfg.n_seqs):
            n = cfg.seqlens[s] - cfg.w
            ref = O.score_window(data["q_win"][s], data["k"][:, cu[s]:cu[s + 1]], cfg.P)
            assert (np.abs(got[:, cu[s]:cu[s] + n] - ref) <= 2e-3 * np.abs(ref)).all()
            assert np.isneginf(got[:, cu[s] + n:cu[s + 1]]).all()
