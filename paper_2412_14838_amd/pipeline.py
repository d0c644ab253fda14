"""Driver of Algorithm 1's layer loop over the C ABI: owns the device buffers, issues the stage calls.

No arithmetic of the method happens here; every step is a dkv_* call.  Buffers (all torch device tensors):
    scores   fp32  [L][Hkv][T]                 A^b, pooled scores of every processed layer
    idx      int32 [L][n_seqs][Hkv][layer_max] ordered candidates of every layer
    counts   int32 [n_seqs][L]                 retained prefix rows per KV head
    budgets_all, hits_all  int32 [L / m][n_seqs][L]   Z' and cnt of every update; `budgets`, `hits`: the latest one's
    kb, vb   [L][n_seqs][Hkv][w + layer_max][d] compressed cache: window rows first, then retained rows;
             layer i of sequence q holds w + counts[q][i] valid rows per head.

Two schedules give identical results: layer by layer (score, select, gather per layer, the paper's order), or
grouped (`group` > 1): the scoring, the selection and the compaction of up to `group` layers are issued in one
call each when the group is full or at the last layer, with one call for the updates that fall inside the group
between selection and compaction (so that only rows the updates keep are copied); the
caller then holds the window queries, K and V of a group's layers until that point.
"""
from __future__ import annotations

import itertools

import torch

from . import dkv

_epochs = itertools.count(1)   # every prefill of every Compressor gets its own non-zero epoch for dkv_rebalance


def default_group(cfg) -> int:
    """Layers per call of the grouped schedule when nothing else is asked for: as many whole update intervals as
    one call of the library takes (all layers, for the benchmark configurations)."""
    most = min(cfg.L, dkv.DKV_MAX_SELECT_LAYERS, dkv.DKV_MAX_UPDATES * cfg.interval)
    return max(most // cfg.interval * cfg.interval, 1)


SCHEDULES = ("dynamic", "fixed", "pyramid", "recent")


class Compressor:
    """schedule: "dynamic" is Algorithm 1 (progressive updates every `interval` layers); "fixed" and "pyramid" score
    and select as Algorithm 1 does but cut every layer to a preset budget instead (no update ever runs);
    "recent" takes sinks + the newest prefix rows as candidates (no scoring) and cuts them to the fixed budget."""

    def __init__(self, cfg, device="cuda", keep_cache=True, desc_override=None, group=1, schedule="dynamic", beta=4,
                 n_sink=4):
        assert schedule in SCHEDULES
        self.cfg = cfg
        self.schedule, self.n_sink = schedule, n_sink
        self.group = max(1, min(int(group), dkv.DKV_MAX_SELECT_LAYERS))
        self._pending = []
        self.on_update = None       # optional host callback(layers_done), called after each update has been issued
        self.device = device
        self.desc = dkv.desc_from_workload(cfg, **(desc_override or {}))
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        L, Hkv, T, d = cfg.L, cfg.Hkv, cfg.total_tokens, cfg.d
        self.slots = cfg.w + cfg.layer_max
        self.cu = torch.tensor(cfg.cu_seqlens, dtype=torch.int32, device=device)
        self.scores = torch.zeros((L, Hkv, T), dtype=torch.float32, device=device)
        self.idx = torch.full((L, cfg.n_seqs, Hkv, cfg.layer_max), -1, dtype=torch.int32, device=device)
        self.counts = torch.zeros((cfg.n_seqs, L), dtype=torch.int32, device=device)
        n_updates = max(1, L // cfg.interval)
        self.budgets_all = torch.zeros((n_updates, cfg.n_seqs, L), dtype=torch.int32, device=device)
        self.hits_all = torch.zeros((n_updates, cfg.n_seqs, L), dtype=torch.int32, device=device)
        self._last_update = 0
        self.epoch = next(_epochs)
        self.keep_cache = keep_cache
        if keep_cache:
            self.kb = torch.zeros((L, cfg.n_seqs, Hkv, self.slots, d), dtype=self.tdtype, device=device)
            self.vb = torch.zeros_like(self.kb)
        self.ws = dkv.alloc_workspace(self.desc, device)
        self.preset = None
        if schedule != "dynamic":
            kind = dkv.DKV_SCHEDULE_PYRAMID if schedule == "pyramid" else dkv.DKV_SCHEDULE_FIXED
            self.preset = torch.tensor(dkv.dkv_layer_budgets(self.desc, kind, beta), dtype=torch.int32, device=device)

    @property
    def budgets(self):
        return self.budgets_all[self._last_update]

    @property
    def hits(self):
        return self.hits_all[self._last_update]

    # one layer of Algorithm 1's loop: score, select, gather, and the update every `interval` layers
    def score(self, layer, q_win, k, stride_token=None, stride_head=None, stream=None):
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_score_window(self.desc, q_win, k, st, sh, self.cu, self.scores[layer], self.cfg.total_tokens, self.ws,
                             stream)

    def score_from_lse(self, layer, q_win, k, lse, stride_token=None, stride_head=None, stream=None):
        """One sweep over K with the caller's row normalisers lse [n_seqs][Hq][w] (natural log, fp32)."""
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_score_window_lse(self.desc, q_win, k, st, sh, self.cu, lse, self.scores[layer], self.cfg.total_tokens,
                                 stream)

    def row_lse(self, lse_out, stride_token=None, stream=None):
        """The normalisers of the layer scored last: lse_out [n_seqs][Hq][w] fp32."""
        st = self.cfg.d if stride_token is None else stride_token
        dkv.dkv_row_lse(self.desc, st, self.cu, lse_out, self.ws, stream)

    def select(self, layer, stream=None):
        dkv.dkv_select_topk(self.desc, layer, self.scores[layer], self.cfg.total_tokens, self.cu, self.idx[layer],
                            self.counts, self.ws, stream)

    def gather(self, layer, k, v, stride_token=None, stride_head=None, stream=None):
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_gather_kv(self.desc, layer, k, v, st, sh, self.cu, self.idx[layer], self.counts, self.kb[layer],
                          self.vb[layer], self.cfg.Hkv * self.slots * d, self.slots * d, stream)

    def select_layers(self, layer_begin, n_layers, stream=None):
        dkv.dkv_select_topk_layers(self.desc, layer_begin, n_layers, self.scores, self.cu, self.idx, self.counts,
                                   self.ws, stream)

    def gather_layers(self, layer_begin, ks, vs, stride_token=None, stride_head=None, stream=None):
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_gather_kv_layers(self.desc, layer_begin, ks, vs, st, sh, self.cu, self.idx, self.counts, self.kb,
                                 self.vb, self.cfg.n_seqs * self.cfg.Hkv * self.slots * d,
                                 self.cfg.Hkv * self.slots * d, self.slots * d, stream)

    def pack(self, capacity_rows=None, stream=None):
        """Tight copy of the final cache: returns (k_packed [rows][d], v_packed, row_offsets int64 [n_seqs*L + 1])."""
        cfg, d = self.cfg, self.cfg.d
        if capacity_rows is None:
            capacity_rows = cfg.n_seqs * cfg.L * cfg.Hkv * self.slots
        kp = torch.zeros((capacity_rows, d), dtype=self.tdtype, device=self.device)
        vp = torch.zeros_like(kp)
        off = torch.zeros(cfg.n_seqs * cfg.L + 1, dtype=torch.int64, device=self.device)
        dkv.dkv_pack_cache(self.desc, self.cu, self.counts, self.kb, self.vb, cfg.n_seqs * cfg.Hkv * self.slots * d,
                           cfg.Hkv * self.slots * d, self.slots * d, kp, vp, capacity_rows, off, stream)
        return kp, vp, off

    def decode_attention(self, layer, q_new, out, lse_out=None, stream=None):
        """Attention of one new token per sequence (q_new [n_seqs][Hq][d]) over layer `layer` of the compressed cache."""
        d = self.cfg.d
        dkv.dkv_decode_attention(self.desc, layer, q_new, self.kb[layer], self.vb[layer], self.cfg.Hkv * self.slots * d,
                                 self.slots * d, self.cu, self.counts, out, lse_out, self.ws, stream)

    def decode_attention_layers(self, layer_begin, n_layers, q_new_all, out_all, lse_all=None, stream=None):
        """The same for n_layers consecutive layers in one call: q_new_all, out_all [n_layers][n_seqs][Hq][d]."""
        d = self.cfg.d
        dkv.dkv_decode_attention_layers(self.desc, layer_begin, n_layers, q_new_all, self.kb, self.vb,
                                        self.cfg.n_seqs * self.cfg.Hkv * self.slots * d, self.cfg.Hkv * self.slots * d,
                                        self.slots * d, self.cu, self.counts, out_all, lse_all, self.ws, stream)

    def _update_slot(self, layers_done):
        return min(max(layers_done // self.cfg.interval - 1, 0), self.budgets_all.shape[0] - 1)

    def rebalance(self, layers_done, stream=None):
        self._last_update = self._update_slot(layers_done)
        dkv.dkv_rebalance(self.desc, layers_done, self.epoch, self.scores, self.cu, self.counts, self.budgets,
                          self.hits, self.ws, stream)

    def rebalance_batch(self, layers_done, n_updates, stream=None):
        """The updates after layers_done, layers_done + interval, ... layers in one call."""
        u0 = self._update_slot(layers_done)
        self._last_update = u0 + n_updates - 1
        dkv.dkv_rebalance_batch(self.desc, layers_done, n_updates, self.epoch, self.scores, self.cu, self.counts,
                                self.budgets_all[u0], self.hits_all[u0], self.cfg.n_seqs * self.cfg.L, self.ws, stream)

    def step(self, layer, q_win, k, v, **strides):
        if layer == 0:
            self.epoch = next(_epochs)      # a new prefill: the updates must not extend the previous one's history
        if self.schedule != "dynamic":
            return self._step_preset(layer, q_win, k, v, **strides)
        if self.group > 1:
            return self._step_grouped(layer, q_win, k, v, **strides)
        self.score(layer, q_win, k, **strides)
        self.select(layer)
        if self.keep_cache:
            self.gather(layer, k, v, **strides)
        if (layer + 1) % self.cfg.interval == 0:
            self._update(layer + 1)

    def apply_budgets(self, n_layers, stream=None):
        dkv.dkv_apply_budgets(self.desc, n_layers, self.preset, self.counts, stream)

    def select_recent(self, layer, stream=None):
        dkv.dkv_select_recent(self.desc, layer, self.n_sink, self.cu, self.idx[layer], self.counts, stream)

    def _step_preset(self, layer, q_win, k, v, **strides):
        # the comparison patterns: the layer's candidates, cut to the preset budget, then the compaction of what is left
        if self.schedule == "recent":
            self.select_recent(layer)
        else:
            self.score(layer, q_win, k, **strides)
            self.select(layer)
        self.apply_budgets(layer + 1)           # a minimum: applying it to the earlier layers again changes nothing
        if self.keep_cache:
            self.gather(layer, k, v, **strides)

    def _update(self, layers_done):
        self.rebalance(layers_done)
        if self.on_update is not None:
            self.on_update(layers_done)

    def score_layers(self, layer_begin, qs, ks, stride_token=None, stride_head=None, stream=None):
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_score_window_layers(self.desc, layer_begin, qs, ks, st, sh, self.cu, self.scores, self.ws, stream)

    def score_layers_from_lse(self, layer_begin, qs, ks, lses, stride_token=None, stride_head=None, stream=None):
        """One sweep over K per layer, several layers per call, with the caller's row normalisers (one tensor
        [n_seqs][Hq][w], natural log, per layer)."""
        d = self.cfg.d
        st = d if stride_token is None else stride_token
        sh = self.cfg.total_tokens * d if stride_head is None else stride_head
        dkv.dkv_score_window_lse_layers(self.desc, layer_begin, qs, ks, st, sh, self.cu, lses, self.scores, self.ws,
                                        stream)

    def _step_grouped(self, layer, q_win, k, v, **strides):
        self._pending.append((layer, k, v, q_win))
        if len(self._pending) < self.group and layer != self.cfg.L - 1:
            return
        pending, self._pending = self._pending, []      # the caller may release K and V of these layers afterwards
        first, n = pending[0][0], len(pending)
        # a layer's selection needs that layer's scores only, and an update touches the layers before its boundary
        # only: one scoring and one selection call for the whole group, one call for the updates that fall inside
        # it, and then the compaction, which copies only the rows those updates have left (a row an update drops
        # never comes back: the later updates only lower the counts)
        self.score_layers(first, [e[3] for e in pending], [e[1] for e in pending], **strides)
        self.select_layers(first, n)
        done = [e[0] + 1 for e in pending if (e[0] + 1) % self.cfg.interval == 0]
        for i in range(0, len(done), dkv.DKV_MAX_UPDATES):      # consecutive boundaries: one call takes several
            part = done[i:i + dkv.DKV_MAX_UPDATES]
            self.rebalance_batch(part[0], len(part))
            if self.on_update is not None:
                for l in part:
                    self._last_update = self._update_slot(l)
                    self.on_update(l)
        if self.keep_cache:
            self.gather_layers(first, [e[1] for e in pending], [e[2] for e in pending], **strides)

    def run(self, layers, overlap=False):
        """layers: sequence of (q_win, k, v) device tensors, one per layer.

        overlap=True issues select / gather / rebalance of layer l on a second stream (default priority), so
        that they run next to the scoring of layer l+1, as they would next to the next layer's forward pass
        in a real prefill; scoring itself stays in layer order on the current stream."""
        if not overlap:
            for l, (q, k, v) in enumerate(layers):
                self.step(l, q, k, v)
            return
        main = torch.cuda.current_stream()
        if getattr(self, "_side", None) is None:
            self._side = torch.cuda.Stream()
        side = self._side
        side.wait_stream(main)
        for l, (q, k, v) in enumerate(layers):
            self.score(l, q, k)
            scored = torch.cuda.Event()
            scored.record(main)
            side.wait_event(scored)
            with torch.cuda.stream(side):
                self.select(l)
                if self.keep_cache:
                    self.gather(l, k, v)
                if (l + 1) % self.cfg.interval == 0:
                    self.rebalance(l + 1)
        main.wait_stream(side)

    def capture(self, layers, overlap=False):
        """Record the whole layer loop over resident inputs into a HIP graph (replay with .replay()).

        The stage calls allocate nothing, never synchronise and clear their scratch with kernels, so the
        loop is capturable as it stands.  Run the loop eagerly once before capturing (first launches set
        kernel attributes)."""
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(layers, overlap=overlap)
        return graph


def to_device(cfg, layer_data, device="cuda"):
    """Upload one make_layer() result in the workload's storage type (values are exactly representable)."""
    tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = {}
    for name in ("q_win", "k", "v"):
        if name in layer_data:
            out[name] = torch.from_numpy(layer_data[name]).to(device=device, dtype=tdtype).contiguous()
    return out
