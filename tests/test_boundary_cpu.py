"""Host-only checks of the C ABI: the library loads, exports what include/dkv.h declares, sizes its
workspace and rejects bad arguments before anything is launched (no GPU needed, no compute calls)."""
import ctypes as C
import os
import re

import pytest

from paper_2412_14838_amd import dkv
from paper_2412_14838_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return dkv.load()


def _good(**kw):
    base = dict(n_layers=4, n_q_heads=4, n_kv_heads=2, head_dim=64, window=16, pool_kernel=7, layer_max=256,
                mean_budget=128, interval=2, dtype=dkv.DKV_F32, n_seqs=1, total_tokens=1024, max_seq_len=1024)
    base.update(kw)
    return dkv.make_desc(**base)


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "dkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(dkv_[a-z_]+)\s*\(", text))
    assert declared == set(dkv.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.dkv_version() == 1
    assert dkv.dkv_status_string(0) == "ok" and "workspace" in dkv.dkv_status_string(dkv.DKV_ERR_WORKSPACE)


def test_descriptor_struct_matches_header():
    text = open(os.path.join(ROOT, "include", "dkv.h")).read()
    body = re.search(r"typedef struct dkv_desc \{(.*?)\} dkv_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|float)\s+(\w+);", body)
    assert [n for _, n in fields] == [n for n, _ in dkv.dkv_desc._fields_]
    assert C.sizeof(dkv.dkv_desc) == 4 * len(fields)


def test_workspace_bytes(lib):
    for cfg in W.standard_configs().values():
        n = dkv.dkv_workspace_bytes(dkv.desc_from_workload(cfg))
        assert n > 0 and n % 256 == 0 and n < 1 << 30
    assert dkv.dkv_workspace_bytes(_good(n_q_heads=5)) == 0


@pytest.mark.parametrize("bad,status", [
    (dict(n_q_heads=5), dkv.DKV_ERR_INVALID_ARG),           # Hq % Hkv
    (dict(pool_kernel=4), dkv.DKV_ERR_INVALID_ARG),         # even pooling kernel
    (dict(pool_kernel=0), dkv.DKV_ERR_INVALID_ARG),
    (dict(window=0), dkv.DKV_ERR_INVALID_ARG),
    (dict(layer_max=0), dkv.DKV_ERR_INVALID_ARG),
    (dict(interval=0), dkv.DKV_ERR_INVALID_ARG),
    (dict(max_seq_len=2048), dkv.DKV_ERR_INVALID_ARG),      # longer than total
    (dict(softmax_scale=-1.0), dkv.DKV_ERR_INVALID_ARG),
    (dict(head_dim=80), dkv.DKV_ERR_UNSUPPORTED),
    (dict(dtype=7), dkv.DKV_ERR_UNSUPPORTED),
    (dict(layer_max=1 << 20), dkv.DKV_ERR_UNSUPPORTED),
    (dict(pool_kernel=129), dkv.DKV_ERR_UNSUPPORTED),
    (dict(n_q_heads=64, n_kv_heads=2, window=32), dkv.DKV_ERR_UNSUPPORTED),   # G * w > 256 rows
])
def test_bad_descriptors_are_rejected(lib, bad, status):
    d = _good(**bad)
    fake = C.c_void_p(0x1000)
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 64 * 1024, fake, fake, 1024, fake, 1 << 30, None) == status
    assert lib.dkv_select_topk(C.byref(d), 0, fake, 1024, fake, fake, fake, fake, 1 << 30, None) == status
    assert lib.dkv_rebalance(C.byref(d), 2, 0, fake, fake, fake, None, None, fake, 1 << 30, None) == status
    assert lib.dkv_gather_kv(C.byref(d), 0, fake, fake, 64, 65536, fake, fake, fake, fake, fake, 2 * 272 * 64,
                             272 * 64, None) == status
    ptrs = (C.c_void_p * 2)(0x1000, 0x2000)
    assert lib.dkv_select_topk_layers(C.byref(d), 0, 2, fake, fake, fake, fake, fake, 1 << 30, None) == status
    assert lib.dkv_gather_kv_layers(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, fake, fake, fake, fake,
                                    2 * 272 * 64, 2 * 272 * 64, 272 * 64, None) == status


def test_long_contexts_size_the_two_level_selection_and_stop_at_the_index_limit(lib):
    """A descriptor whose rows can pass 32768 candidate positions asks for the candidate lists of the two-level
    selection (layers of a call x rows x segments x layer_max x 8 bytes); score tensors of more than 2^31 elements
    (the index arithmetic of the update is 32-bit per layer block) are refused with DKV_ERR_UNSUPPORTED."""
    kw = dict(head_dim=128, dtype=dkv.DKV_BF16, n_q_heads=32, n_kv_heads=8, window=32, layer_max=2048, mean_budget=512,
              n_layers=32, interval=4)
    short = dkv.dkv_workspace_bytes(_good(total_tokens=32768 + 32, max_seq_len=32768 + 32, **kw))
    longer = dkv.dkv_workspace_bytes(_good(total_tokens=32768 + 33, max_seq_len=32768 + 33, **kw))
    assert longer - short >= 32 * 8 * 2 * 2048 * 8 and longer - short < 32 * 8 * 2 * 2048 * 8 + (1 << 20)
    million = _good(total_tokens=1 << 20, max_seq_len=1 << 20, **kw)
    assert dkv.dkv_workspace_bytes(million) > 32 * 8 * 32 * 2048 * 8
    fake = C.c_void_p(0x1000)
    # 32 layers x 8 heads x 2^23 tokens = 2^31 elements: the last size that is accepted; one more layer is not
    edge = _good(total_tokens=1 << 23, max_seq_len=1 << 23, **kw)
    assert dkv.dkv_workspace_bytes(edge) > 0
    over = _good(total_tokens=1 << 23, max_seq_len=1 << 23, **dict(kw, n_layers=36))
    assert dkv.dkv_workspace_bytes(over) == 0
    assert lib.dkv_select_topk(C.byref(over), 0, fake, 1 << 23, fake, fake, fake, fake, 1 << 40, None) == dkv.DKV_ERR_UNSUPPORTED
    assert lib.dkv_rebalance(C.byref(over), 4, 0, fake, fake, fake, None, None, fake, 1 << 40, None) == dkv.DKV_ERR_UNSUPPORTED
    assert lib.dkv_score_window(C.byref(over), fake, fake, 128, 128 << 23, fake, fake, 1 << 23, fake, 1 << 40, None) == dkv.DKV_ERR_UNSUPPORTED


def test_bad_call_arguments_are_rejected(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    odd = C.c_void_p(0x1004)
    inv, wsp = dkv.DKV_ERR_INVALID_ARG, dkv.DKV_ERR_WORKSPACE
    # null pointers
    assert lib.dkv_score_window(C.byref(d), None, fake, 64, 65536, fake, fake, 1024, fake, need, None) == inv
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 65536, None, fake, 1024, fake, need, None) == inv
    assert lib.dkv_select_topk(C.byref(d), 0, None, 1024, fake, fake, fake, fake, need, None) == inv
    assert lib.dkv_rebalance(C.byref(d), 2, 0, fake, fake, None, None, None, fake, need, None) == inv
    assert lib.dkv_gather_kv(C.byref(d), 0, fake, None, 64, 65536, fake, fake, fake, fake, fake, 2 * 272 * 64, 272 * 64,
                             None) == inv
    assert lib.dkv_workspace_bytes(None) == 0
    # misaligned pointers / strides
    assert lib.dkv_score_window(C.byref(d), fake, odd, 64, 65536, fake, fake, 1024, fake, need, None) == inv
    assert lib.dkv_score_window(C.byref(d), fake, fake, 65, 65536, fake, fake, 1024, fake, need, None) == inv
    assert lib.dkv_score_window(C.byref(d), fake, fake, 32, 65536, fake, fake, 1024, fake, need, None) == inv
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 65536, fake, fake, 1000, fake, need, None) == inv
    # workspace missing, too small or misaligned
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 65536, fake, fake, 1024, None, need, None) == wsp
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 65536, fake, fake, 1024, fake, need - 1, None) == wsp
    assert lib.dkv_score_window(C.byref(d), fake, fake, 64, 65536, fake, fake, 1024, C.c_void_p(0x1010), need, None) == wsp
    assert lib.dkv_rebalance(C.byref(d), 2, 0, fake, fake, fake, None, None, fake, 16, None) == wsp
    # layer / layers_done out of range or not a multiple of the interval
    assert lib.dkv_select_topk(C.byref(d), 4, fake, 1024, fake, fake, fake, fake, need, None) == inv
    assert lib.dkv_select_topk(C.byref(d), -1, fake, 1024, fake, fake, fake, fake, need, None) == inv
    for bad_l in (0, 1, 3, 6):
        assert lib.dkv_rebalance(C.byref(d), bad_l, 0, fake, fake, fake, None, None, fake, need, None) == inv
    # output block too small for window + layer_max rows
    assert lib.dkv_gather_kv(C.byref(d), 0, fake, fake, 64, 65536, fake, fake, fake, fake, fake, 2 * 100 * 64, 100 * 64,
                             None) == inv
    assert lib.dkv_gather_kv(C.byref(d), 9, fake, fake, 64, 65536, fake, fake, fake, fake, fake, 2 * 272 * 64, 272 * 64,
                             None) == inv


def test_layer_batched_calls_reject_bad_ranges(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    ptrs = (C.c_void_p * 9)(*([0x1000] * 9))
    bad = (C.c_void_p * 2)(0x1000, 0)          # a null layer pointer
    odd = (C.c_void_p * 2)(0x1000, 0x1008)     # a misaligned layer pointer
    sl, sq, sh = 2 * 272 * 64, 2 * 272 * 64, 272 * 64
    for begin, n in ((0, 0), (0, 9), (3, 2), (-1, 1), (4, 1)):
        assert lib.dkv_select_topk_layers(C.byref(d), begin, n, fake, fake, fake, fake, fake, need, None) == inv
        assert lib.dkv_gather_kv_layers(C.byref(d), begin, n, ptrs, ptrs, 64, 65536, fake, fake, fake, fake, fake,
                                        sl, sq, sh, None) == inv
    assert lib.dkv_select_topk_layers(C.byref(d), 0, 2, None, fake, fake, fake, fake, need, None) == inv
    assert lib.dkv_select_topk_layers(C.byref(d), 0, 2, fake, fake, fake, fake, fake, need - 1, None) == dkv.DKV_ERR_WORKSPACE
    for arr in (bad, odd):
        assert lib.dkv_gather_kv_layers(C.byref(d), 0, 2, arr, ptrs, 64, 65536, fake, fake, fake, fake, fake,
                                        sl, sq, sh, None) == inv
        assert lib.dkv_gather_kv_layers(C.byref(d), 0, 2, ptrs, arr, 64, 65536, fake, fake, fake, fake, fake,
                                        sl, sq, sh, None) == inv
    assert lib.dkv_gather_kv_layers(C.byref(d), 0, 2, None, ptrs, 64, 65536, fake, fake, fake, fake, fake,
                                    sl, sq, sh, None) == inv
    # layer stride smaller than one layer's block
    assert lib.dkv_gather_kv_layers(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, fake, fake, fake, fake,
                                    sq - 64, sq, sh, None) == inv


def test_batched_updates_validate_their_arguments(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    call = lib.dkv_rebalance_batch
    big = d.n_seqs * d.n_layers
    assert call(C.byref(d), d.interval, 0, 0, fake, fake, fake, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval, dkv.DKV_MAX_UPDATES + 1, 0, fake, fake, fake, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval + 1, 1, 0, fake, fake, fake, fake, fake, big, fake, need, None) == inv      # not a boundary
    assert call(C.byref(d), 0, 1, 0, fake, fake, fake, fake, fake, big, fake, need, None) == inv
    last = d.n_layers // d.interval * d.interval
    assert call(C.byref(d), last, 2, 0, fake, fake, fake, fake, fake, big, fake, need, None) == inv                # runs past L
    assert call(C.byref(d), d.interval, 2, 0, fake, fake, fake, fake, fake, big - 1, fake, need, None) == inv      # outputs overlap
    assert call(C.byref(d), d.interval, 2, 0, None, fake, fake, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval, 2, 0, fake, None, fake, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval, 2, 0, fake, fake, None, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval, 2, 0, C.c_void_p(0x1004), fake, fake, fake, fake, big, fake, need, None) == inv
    assert call(C.byref(d), d.interval, 2, 0, fake, fake, fake, fake, fake, big, None, need, None) == dkv.DKV_ERR_WORKSPACE
    assert call(C.byref(d), d.interval, 2, 0, fake, fake, fake, fake, fake, big, fake, need - 1, None) == dkv.DKV_ERR_WORKSPACE


def test_layer_batched_scoring_rejects_bad_ranges_and_pointers(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    ptrs = (C.c_void_p * 9)(*([0x1000] * 9))
    bad = (C.c_void_p * 2)(0x1000, 0)          # a null layer pointer
    odd = (C.c_void_p * 2)(0x1000, 0x1008)     # a misaligned layer pointer
    call = lib.dkv_score_window_layers
    for begin, n in ((0, 0), (0, 9), (3, 2), (-1, 1), (4, 1)):
        assert call(C.byref(d), begin, n, ptrs, ptrs, 64, 65536, fake, fake, fake, need, None) == inv
    for arr in (bad, odd):
        assert call(C.byref(d), 0, 2, arr, ptrs, 64, 65536, fake, fake, fake, need, None) == inv
        assert call(C.byref(d), 0, 2, ptrs, arr, 64, 65536, fake, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, None, ptrs, 64, 65536, fake, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, None, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, None, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, fake, None, need, None) == dkv.DKV_ERR_WORKSPACE
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, fake, fake, need - 1, None) == dkv.DKV_ERR_WORKSPACE
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 63, 65536, fake, fake, fake, need, None) == inv     # rows overlap
    assert call(None, 0, 2, ptrs, ptrs, 64, 65536, fake, fake, fake, need, None) == inv


def test_layer_batched_single_sweep_validates_its_arguments(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    ptrs = (C.c_void_p * 9)(*([0x1000] * 9))
    bad = (C.c_void_p * 2)(0x1000, 0)          # a null layer pointer
    call = lib.dkv_score_window_lse_layers
    for begin, n in ((0, 0), (0, 9), (3, 2), (-1, 1), (4, 1)):
        assert call(C.byref(d), begin, n, ptrs, ptrs, 64, 65536, fake, ptrs, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, bad, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, None, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, bad, ptrs, 64, 65536, fake, ptrs, fake, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, ptrs, None, fake, need, None) == inv
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, ptrs, fake, None, need, None) == dkv.DKV_ERR_WORKSPACE
    assert call(C.byref(d), 0, 2, ptrs, ptrs, 64, 65536, fake, ptrs, fake, fake, need - 1, None) == dkv.DKV_ERR_WORKSPACE


def test_lse_calls_validate_their_arguments(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv, wsp = dkv.DKV_ERR_INVALID_ARG, dkv.DKV_ERR_WORKSPACE
    assert lib.dkv_score_window_lse(C.byref(d), fake, fake, 64, 65536, fake, None, fake, 1024, None) == inv   # no lse
    assert lib.dkv_score_window_lse(C.byref(d), None, fake, 64, 65536, fake, fake, fake, 1024, None) == inv
    assert lib.dkv_score_window_lse(C.byref(d), fake, fake, 64, 65536, fake, fake, None, 1024, None) == inv
    assert lib.dkv_score_window_lse(C.byref(d), fake, fake, 64, 65536, fake, fake, fake, 1000, None) == inv
    assert lib.dkv_score_window_lse(C.byref(_good(pool_kernel=2)), fake, fake, 64, 65536, fake, fake, fake, 1024,
                                    None) == inv
    assert lib.dkv_row_lse(C.byref(d), 64, fake, None, fake, need, None) == inv
    assert lib.dkv_row_lse(C.byref(d), 64, None, fake, fake, need, None) == inv
    assert lib.dkv_row_lse(C.byref(d), 64, fake, fake, None, need, None) == wsp
    assert lib.dkv_row_lse(C.byref(d), 64, fake, fake, fake, need - 1, None) == wsp
    assert lib.dkv_row_lse(None, 64, fake, fake, fake, need, None) == inv


def test_pack_cache_validates_its_arguments(lib):
    d = _good()
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    sl, sq, sh = 2 * 272 * 64, 2 * 272 * 64, 272 * 64
    ok_args = [fake, fake, fake, fake, sl, sq, sh, fake, fake, 1000, fake, None]
    for i in (0, 1, 2, 3, 7, 8, 10):          # each required pointer in turn
        a = list(ok_args)
        a[i] = None
        assert lib.dkv_pack_cache(C.byref(d), *a) == inv
    a = list(ok_args); a[10] = C.c_void_p(0x1004)          # offsets not 8-byte aligned
    assert lib.dkv_pack_cache(C.byref(d), *a) == inv
    a = list(ok_args); a[6] = sh - 64                      # head stride smaller than a block
    assert lib.dkv_pack_cache(C.byref(d), *a) == inv
    a = list(ok_args); a[9] = -1
    assert lib.dkv_pack_cache(C.byref(d), *a) == inv
    assert lib.dkv_pack_cache(C.byref(_good(interval=0)), *ok_args) == inv


def test_decode_attention_validates_its_arguments(lib):
    d = _good()
    need = dkv.dkv_workspace_bytes(d)
    fake = C.c_void_p(0x1000)
    inv, wsp = dkv.DKV_ERR_INVALID_ARG, dkv.DKV_ERR_WORKSPACE
    sq, sh = 2 * 272 * 64, 272 * 64
    ok = [0, fake, fake, fake, sq, sh, fake, fake, fake, None, fake, need, None]
    for i in (1, 2, 3, 6, 7, 8):                 # each required pointer in turn (lse_out may be null)
        a = list(ok)
        a[i] = None
        assert lib.dkv_decode_attention(C.byref(d), *a) == inv
    for layer in (-1, 4):
        a = list(ok); a[0] = layer
        assert lib.dkv_decode_attention(C.byref(d), *a) == inv
    a = list(ok); a[5] = sh - 64                 # head stride smaller than a block
    assert lib.dkv_decode_attention(C.byref(d), *a) == inv
    a = list(ok); a[10] = None
    assert lib.dkv_decode_attention(C.byref(d), *a) == wsp
    a = list(ok); a[11] = need - 1
    assert lib.dkv_decode_attention(C.byref(d), *a) == wsp
    wide = _good(n_q_heads=34, n_kv_heads=2, window=4)        # 17 query heads per KV head
    assert lib.dkv_decode_attention(C.byref(wide), *ok[:11], dkv.dkv_workspace_bytes(wide), None) == dkv.DKV_ERR_UNSUPPORTED
    # the layer-batched form
    sl = 2 * 272 * 64
    okl = [0, 4, fake, fake, fake, sl, sq, sh, fake, fake, fake, None, fake, need, None]
    call = lib.dkv_decode_attention_layers
    for i in (2, 3, 4, 8, 9, 10):
        a = list(okl)
        a[i] = None
        assert call(C.byref(d), *a) == inv
    for begin, n in ((0, 0), (0, 5), (3, 2), (-1, 1), (4, 1)):
        a = list(okl); a[0], a[1] = begin, n
        assert call(C.byref(d), *a) == inv
    a = list(okl); a[5] = sl - 64                # layer stride smaller than one layer's blocks
    assert call(C.byref(d), *a) == inv
    a = list(okl); a[12] = None
    assert call(C.byref(d), *a) == wsp
    a = list(okl); a[13] = need - 1
    assert call(C.byref(d), *a) == wsp
    assert call(C.byref(wide), *okl[:13], dkv.dkv_workspace_bytes(wide), None) == dkv.DKV_ERR_UNSUPPORTED


def test_fixed_pattern_schedules_match_the_oracle_and_validate(lib):
    """dkv_layer_budgets is host-only: its budgets equal the oracle's for both schedules over a sweep of shapes
    (including a hi that hits the per-layer maximum, beta = 1 and L = 1), and bad arguments are rejected."""
    from oracle import dkv_oracle as O
    for L in (1, 2, 4, 7, 28, 32):
        for mean, layer_max in ((128, 256), (512, 2048), (64, 100), (7, 9), (1, 1)):
            d = _good(n_layers=L, mean_budget=mean, layer_max=layer_max, interval=1)
            assert dkv.dkv_layer_budgets(d, dkv.DKV_SCHEDULE_FIXED) == O.fixed_layer_budgets(L, mean).tolist()
            for beta in (1, 2, 4, 9):
                assert dkv.dkv_layer_budgets(d, dkv.DKV_SCHEDULE_PYRAMID, beta) == \
                    O.pyramid_layer_budgets(L, mean, layer_max, beta).tolist(), (L, mean, layer_max, beta)
    d = _good()
    out = (C.c_int32 * 4)()
    fake = C.c_void_p(0x1000)
    inv = dkv.DKV_ERR_INVALID_ARG
    assert lib.dkv_layer_budgets(C.byref(d), 2, 4, out) == inv            # unknown schedule
    assert lib.dkv_layer_budgets(C.byref(d), dkv.DKV_SCHEDULE_PYRAMID, 0, out) == inv
    assert lib.dkv_layer_budgets(C.byref(d), dkv.DKV_SCHEDULE_FIXED, 4, None) == inv
    assert lib.dkv_layer_budgets(C.byref(_good(interval=0)), dkv.DKV_SCHEDULE_FIXED, 4, out) == inv
    assert lib.dkv_apply_budgets(C.byref(d), 4, None, fake, None) == inv
    assert lib.dkv_apply_budgets(C.byref(d), 4, fake, None, None) == inv
    for n in (0, 5):
        assert lib.dkv_apply_budgets(C.byref(d), n, fake, fake, None) == inv
    assert lib.dkv_select_recent(C.byref(d), 0, 4, None, fake, fake, None) == inv
    assert lib.dkv_select_recent(C.byref(d), 0, -1, fake, fake, fake, None) == inv
    assert lib.dkv_select_recent(C.byref(d), 4, 4, fake, fake, fake, None) == inv
    assert lib.dkv_select_recent(C.byref(_good(pool_kernel=2)), 0, 4, fake, fake, fake, None) == inv


def test_score_path_and_the_token_stride_limit(lib):
    """The matrix-core kernels form key-row offsets in 32 bits: a token stride whose product with the largest row
    index of a chunk would pass 2^32 bytes must take the vector-ALU kernels (dkv_score_path tells which)."""
    bf = _good(head_dim=128, dtype=dkv.DKV_BF16, n_q_heads=8, n_kv_heads=2, window=32)
    assert lib.dkv_score_path(C.byref(bf), 128) == 1
    assert lib.dkv_score_path(C.byref(bf), 8 * 128) == 1                   # token-major, 8 KV heads
    limit_elems = (1 << 32) // (4096 + 64 + 256) // 2                      # bytes -> bf16 elements
    assert lib.dkv_score_path(C.byref(bf), limit_elems // 8 * 8) == 1
    assert lib.dkv_score_path(C.byref(bf), (limit_elems // 8 + 1) * 8) == 0
    assert lib.dkv_score_path(C.byref(bf), 1 << 22) == 0
    assert lib.dkv_score_path(C.byref(_good()), 64) == 0                   # fp32: vector ALU
    assert lib.dkv_score_path(C.byref(_good(head_dim=64, dtype=dkv.DKV_BF16)), 64) == 0
    assert lib.dkv_score_path(C.byref(bf), 100) == dkv.DKV_ERR_INVALID_ARG  # rows overlap
    assert lib.dkv_score_path(None, 128) == dkv.DKV_ERR_INVALID_ARG
    assert lib.dkv_score_path(C.byref(_good(n_kv_heads=2048, n_q_heads=2048)), 64) == dkv.DKV_ERR_UNSUPPORTED


def test_static_scratch_entry_rejects_what_does_not_fit(lib):
    """dkv_score_window_static validates like dkv_score_window and refuses, before anything is launched, a problem
    whose row statistics do not fit its fixed array."""
    fake = C.c_void_p(0x1000)
    limit = dkv.dkv_static_scratch_limit()
    assert limit == 8 << 20
    big = _good(head_dim=128, dtype=dkv.DKV_BF16, n_q_heads=32, n_kv_heads=8, window=32, total_tokens=1 << 19,
                max_seq_len=1 << 19, n_layers=2)
    need = ((1 << 19) // 256 + 1) * 8 * 128 * 8
    assert need > limit
    assert lib.dkv_score_window_static(C.byref(big), fake, fake, 128, 128 << 19, fake, fake, 1 << 19, None) == dkv.DKV_ERR_UNSUPPORTED
    d = _good()
    assert lib.dkv_score_window_static(C.byref(d), None, fake, 64, 65536, fake, fake, 1024, None) == dkv.DKV_ERR_INVALID_ARG
    assert lib.dkv_score_window_static(C.byref(d), fake, fake, 64, 65536, fake, fake, 1000, None) == dkv.DKV_ERR_INVALID_ARG
    assert lib.dkv_score_window_static(C.byref(_good(pool_kernel=2)), fake, fake, 64, 65536, fake, fake, 1024, None) == dkv.DKV_ERR_INVALID_ARG


def test_binding_raises_on_error():
    d = _good(pool_kernel=2)
    with pytest.raises(dkv.DkvError):
        dkv._check(dkv.load().dkv_select_topk(C.byref(d), 0, None, 0, None, None, None, None, 0, None), "dkv_select_topk")
