"""Prediction interval with neighbour fetching (Sec. 3.4), as a harness-level loop over the
C-ABI entry points.  No arithmetic happens here: every step of the path is a library call.

Step t sees the first ``N0 + t`` rows of the cache.  On prediction steps (``t % P == 0``) the
newly appended keys are projected, the whole cache is scored, the top-k selection is made and
attention runs on it; the selection widened by its neighbours is kept.  On the other steps
attention runs on the kept list plus the dense tail of rows appended since the prediction (the
local window is refreshed every step), and nothing else is touched.

With ``buffered=True`` the widened selection is migrated into per-query-head buffers on the
prediction step (the paper's Important Buffer, Sec. 3.3) and the other steps attend over the
buffers plus the dense tail; the fused form gathers the rows from the cache on every step.

With ``headless=True`` the importance has no head dimension (Appendix "Additional Efficiency
Evaluation"): ``Kimp`` is ``[B][1][Ncap][d']``, ``q_imp`` is ``[B][1][d']``, one list per batch
element is selected, widened and attended by every head.
"""
from __future__ import annotations

import torch

from . import binding as tb


class IntervalDecoder:
    def __init__(self, K, V, W, Kimp, Hq: int, k: int, P: int, radius: int, sink: int = 0, window: int = 0,
                 sm_scale: float = 1.0, score_scale: float = 1.0, mode: int = 0, expand_on_predict: bool = False,
                 buffered: bool = False, headless: bool = False):
        self.K, self.V, self.W, self.Kimp = K, V, W, Kimp
        self.B, self.Hkv, self.Ncap, self.D = K.shape
        self.Hq, self.k, self.P, self.radius = Hq, k, P, radius
        self.sink, self.window, self.sm_scale, self.score_scale = sink, window, sm_scale, score_scale
        self.mode, self.expand_on_predict = mode, expand_on_predict
        self.headless = headless
        assert not (headless and buffered), "the buffers are per query head"
        dev = K.device
        B = self.B
        Hl = 1 if headless else Hq  # heads that carry a list of their own
        self.sel_cap = sink + k + window
        mult = (2 * radius + 1) if mode == 0 else 2
        self.exp_cap = min(self.Ncap, mult * self.sel_cap)
        self.scores = torch.empty((B, Hl, (self.Ncap + 3) // 4 * 4), dtype=torch.float32, device=dev)
        self.idx = torch.zeros((B, Hl, self.sel_cap), dtype=torch.int32, device=dev)
        self.cnt = torch.zeros((B, Hl), dtype=torch.int32, device=dev)
        self.exp_idx = torch.zeros((B, Hl, self.exp_cap), dtype=torch.int32, device=dev)
        self.exp_cnt = torch.zeros((B, Hl), dtype=torch.int32, device=dev)
        self.out = torch.empty((B, Hq, self.D), dtype=torch.float32, device=dev)
        self.lse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
        desc = tb.make_desc(self.Ncap, Hq, K=K, V=V, Kimp=None if headless else Kimp, Dimp=Kimp.shape[3])
        self.ws = tb.new_workspace(tb.TB_OP_DECODE_STEP, desc, self.exp_cap + P)
        if headless:
            self.sel_ws = tb.new_workspace(tb.TB_OP_SELECT, tb.make_desc(self.Ncap, 1, Kimp=Kimp), self.sel_cap)
        self.N_pred = None
        self.projected_upto = None
        self.buffered = buffered
        if buffered:
            self.Kbuf = torch.empty((B, Hq, self.exp_cap, self.D), dtype=K.dtype, device=dev)
            self.Vbuf = torch.empty_like(self.Kbuf)

    def _step_headless(self, t: int, N_t: int, q: torch.Tensor, q_imp: torch.Tensor):
        desc = tb.make_desc(N_t, self.Hq, K=self.K, V=self.V, Dimp=self.Kimp.shape[3])
        attend = tb.tb_sparse_decode_attn_shared
        if t % self.P == 0:
            # the importance head (the caller keeps its keys up to date: how they are derived from
            # the layer's state is not given for this variant, so no projection happens here)
            d1 = tb.make_desc(N_t, 1, Kimp=self.Kimp)
            tb.tb_score(d1, q_imp, self.Kimp, self.score_scale, self.scores)
            tb.tb_select_topk(d1, self.scores, self.k, self.sink, self.window, self.idx, self.cnt, self.sel_ws)
            tb.tb_expand_neighbors(self.B, 1, N_t, self.radius, self.mode, self.idx, self.cnt, self.exp_idx,
                                   self.exp_cnt)
            self.N_pred = N_t
            if self.expand_on_predict:
                attend(desc, q, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap, self.sm_scale, self.out,
                       self.lse, self.ws)
            else:
                attend(desc, q, self.K, self.V, self.idx, self.cnt, self.sel_cap, self.sm_scale, self.out, self.lse,
                       self.ws)
        else:
            attend(desc, q, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap, self.sm_scale, self.out,
                   self.lse, self.ws, tail_begin=self.N_pred, tail_end=N_t)
        return self.out, self.lse

    def step(self, t: int, N_t: int, q: torch.Tensor, q_imp: torch.Tensor):
        """Returns (out, lse) views valid until the next call."""
        if self.headless:
            return self._step_headless(t, N_t, q, q_imp)
        desc = tb.make_desc(N_t, self.Hq, K=self.K, V=self.V, Kimp=self.Kimp)
        if t % self.P == 0:
            if self.projected_upto is None:
                self.projected_upto = N_t  # the caller projected the post-prefill cache
            if self.projected_upto < N_t:  # batched deferred projection of the rows appended since
                tb.tb_project_keys(desc, self.K, self.W, self.Kimp, self.projected_upto, N_t)
                self.projected_upto = N_t
            tb.tb_decode_step(desc, q_imp, self.Kimp, self.score_scale, q, self.K, self.V, self.k, self.sink,
                              self.window, self.sm_scale, self.scores, self.idx, self.cnt, self.out, self.lse, self.ws)
            tb.tb_expand_neighbors(self.B, self.Hq, N_t, self.radius, self.mode, self.idx, self.cnt, self.exp_idx,
                                   self.exp_cnt)
            self.N_pred = N_t
            if self.buffered:
                tb.tb_gather_kv(desc, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap, self.Kbuf, self.Vbuf)
            if self.expand_on_predict:
                tb.tb_sparse_decode_attn(desc, q, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap,
                                         self.sm_scale, self.out, self.lse, self.ws)
        elif self.buffered:
            tb.tb_buffered_decode_attn(desc, q, self.Kbuf, self.Vbuf, self.exp_cnt, self.exp_cap, self.K, self.V,
                                       self.sm_scale, self.out, self.lse, self.ws, tail_begin=self.N_pred,
                                       tail_end=N_t)
        else:
            tb.tb_sparse_decode_attn(desc, q, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap,
                                     self.sm_scale, self.out, self.lse, self.ws, tail_begin=self.N_pred, tail_end=N_t)
        return self.out, self.lse


class RingLayoutDecoder:
    """The three physical buffers of Sec. 3.3 "Inference Setup", driven through the C-ABI calls.

    Sink Buffer and Local Window ring are one allocation ``aux`` of ``sink + ring`` rows per KV
    head (rows ``[0, sink)``: the first tokens, copied once; rows ``[sink, sink + ring)``: the
    circular queue of the newest tokens, slot ``(t - 1) % ring`` for the token appended before
    step t); the Important Buffer holds, per query head, the widened selection without its sink
    and window entries (``tb_gather_important``).  Every step attends over Important Buffer,
    Sink Buffer and ring (``tb_buffered_decode_attn`` with the dense range over ``aux``): no row
    of the big cache is gathered outside prediction steps.

    Projection is deferred as the paper describes: starting from the post-prefill state (all
    keys projected, the ring empty) nothing is projected until the ring's head is back at slot
    0, then the ``ring`` keys in the ring are projected in one batch -- read from the ring --
    and appended to the projected-key cache.  Tokens in the ring are attended without a score,
    so the selection never needs a projected key that does not exist yet.

    Moving the model's new K/V row into the ring (and the first ``sink`` rows into the Sink
    Buffer) is data arrival, done here with a plain device copy; everything that computes is a
    library call.
    """

    def __init__(self, K, V, W, Kimp, Hq: int, k: int, P: int, radius: int, ring: int, sink: int = 0,
                 sm_scale: float = 1.0, score_scale: float = 1.0, mode: int = 0):
        assert ring >= P, "the ring must cover a prediction interval"
        self.K, self.V, self.W, self.Kimp = K, V, W, Kimp
        self.B, self.Hkv, self.Ncap, self.D = K.shape
        self.Hq, self.k, self.P, self.radius, self.ring, self.sink = Hq, k, P, radius, ring, sink
        self.sm_scale, self.score_scale, self.mode = sm_scale, score_scale, mode
        dev, B = K.device, self.B
        self.aux_K = torch.zeros((B, self.Hkv, sink + ring, self.D), dtype=K.dtype, device=dev)
        self.aux_V = torch.zeros_like(self.aux_K)
        self.aux_K[:, :, :sink].copy_(K[:, :, :sink])
        self.aux_V[:, :, :sink].copy_(V[:, :, :sink])
        self.sel_cap = sink + k + ring
        mult = (2 * radius + 1) if mode == 0 else 2
        self.exp_cap = min(self.Ncap, mult * self.sel_cap)
        self.scores = torch.empty((B, Hq, (self.Ncap + 3) // 4 * 4), dtype=torch.float32, device=dev)
        self.idx = torch.zeros((B, Hq, self.sel_cap), dtype=torch.int32, device=dev)
        self.cnt = torch.zeros((B, Hq), dtype=torch.int32, device=dev)
        self.exp_idx = torch.zeros((B, Hq, self.exp_cap), dtype=torch.int32, device=dev)
        self.exp_cnt = torch.zeros((B, Hq), dtype=torch.int32, device=dev)
        self.imp_cnt = torch.zeros((B, Hq), dtype=torch.int32, device=dev)
        self.Kbuf = torch.empty((B, Hq, self.exp_cap, self.D), dtype=K.dtype, device=dev)
        self.Vbuf = torch.empty_like(self.Kbuf)
        self.out = torch.empty((B, Hq, self.D), dtype=torch.float32, device=dev)
        self.lse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
        self.sel_ws = tb.new_workspace(tb.TB_OP_SELECT, tb.make_desc(self.Ncap, Hq, K=K, V=V, Kimp=Kimp), self.sel_cap)
        self.ws = tb.new_workspace(tb.TB_OP_ATTN, tb.make_desc(sink + ring, Hq, K=self.aux_K, V=self.aux_V),
                                   self.exp_cap + sink + ring)
        self.projections = 0  # batched projections done (one per wrap of the ring)

    def step(self, t: int, N_t: int, q: torch.Tensor, q_imp: torch.Tensor):
        """Step t sees the first N_t = N0 + t rows of the cache.  Returns (out, lse) views."""
        S, R = self.sink, self.ring
        if t > 0:  # the token appended before this step arrives in the ring
            slot = (t - 1) % R
            self.aux_K[:, :, S + slot].copy_(self.K[:, :, N_t - 1])
            self.aux_V[:, :, S + slot].copy_(self.V[:, :, N_t - 1])
            if t % R == 0:
                # the head is back at slot 0: slot i holds token N_t - R + i; project the R keys of
                # the ring in one batch and append them to the projected-key cache
                ring_K = self.aux_K[:, :, S:S + R]
                kimp_rows = self.Kimp[:, :, N_t - R:N_t]
                tb.tb_project_keys(tb.make_desc(R, self.Hq, K=ring_K, Kimp=kimp_rows), ring_K, self.W, kimp_rows, 0, R)
                self.projections += 1
        W_t = min(R, t)  # tokens in the ring
        if t % self.P == 0:
            desc = tb.make_desc(N_t, self.Hq, K=self.K, V=self.V, Kimp=self.Kimp)
            tb.tb_score(desc, q_imp, self.Kimp, self.score_scale, self.scores)
            tb.tb_select_topk(desc, self.scores, self.k, S, W_t, self.idx, self.cnt, self.sel_ws)
            tb.tb_expand_neighbors(self.B, self.Hq, N_t, self.radius, self.mode, self.idx, self.cnt, self.exp_idx,
                                   self.exp_cnt)
            # migration into the Important Buffer: the widened list without its sink and window entries
            tb.tb_gather_important(desc, self.K, self.V, self.exp_idx, self.exp_cnt, self.exp_cap, min(S, N_t), W_t,
                                   self.Kbuf, self.Vbuf, self.imp_cnt)
        aux = tb.make_desc(S + W_t, self.Hq, K=self.aux_K, V=self.aux_V)
        tb.tb_buffered_decode_attn(aux, q, self.Kbuf, self.Vbuf, self.imp_cnt, self.exp_cap, self.aux_K, self.aux_V,
                                   self.sm_scale, self.out, self.lse, self.ws, tail_begin=0, tail_end=S + W_t)
        return self.out, self.lse
