"""Decode-step driver over the C ABI: model-level setup and the per-layer call sequence.

Everything the method computes happens inside libinfinigen_hip (ig_skew_offline, ig_partial_index,
ig_wq_build, ig_slab_build, ig_speculate, ig_gather_kv, ig_sparse_attention).  This module only
allocates tensors, draws the synthetic model state that surrounds the path (weights, KV cache,
layer inputs, the layer's real query) and issues the calls in the order of the paper's decode
stage (Section 4.3, Fig. 3(d)): rehearsal of layer i+1 -> prefetch of its K/V rows -> attention.
"""
from __future__ import annotations

import math

import numpy as np
import torch

import ig_workloads as wl
from . import binding as ig


class Rehearsal:
    """State of `layers` decoder layers of one workload and the hot-path call sequence over them."""

    def __init__(self, ctx: ig.Context, w: wl.Workload, gain: float | None = None,
                 layers: int | None = None, host_layers: int = 4, sets: int = 2,
                 extra_tokens: int = 0, log=lambda *a: None, offline_from: "Rehearsal | None" = None):
        self.ctx, self.w = ctx, w
        self.L = layers or w.layers
        self.gain = w.gain if gain is None else gain
        dev = "cuda"
        tdt = torch.float32 if w.dtype == "f32" else torch.float16
        self.tdt = tdt
        self.N_cap = w.N + extra_tokens      # room for the tokens a decode loop appends
        if offline_from is not None:
            # same model (weights, skewing, partial index, weight blob), other layers / capacity
            o_ = offline_from
            assert o_.w is w and o_.gain == self.gain
            for name in ("A", "idx_host", "r", "idx", "W_host", "wq", "A_p", "pos", "_Wd"):
                setattr(self, name, getattr(o_, name))
            self.desc = ig.IgDesc(B=w.B, H=w.H, d=w.d, r=self.r, N=w.N, N_cap=self.N_cap,
                                  dtype=o_.desc.dtype, scale=o_.desc.scale, alpha=w.alpha,
                                  rope=o_.desc.rope)
            ctx.ig_reserve(self.desc)
            self._build_layers(host_layers, sets, log)
            return

        # ---- offline: skewing (Section 4.2) on the calibration queries ----
        Wq = wl.projection_weight(w, "Wq")
        Xcal = wl.calibration_input(w)
        Qcal = Xcal @ Wq
        if w.rope:
            Qcal = ig.ig_rope_rows(Qcal.reshape(w.n_cal, w.H, w.d), np.arange(w.n_cal),
                                   ctx=ctx).reshape(w.n_cal, w.D)
        log("weights drawn")
        sk = ig.ig_skew_offline(Wq, None, Qcal, w.H, ctx=ctx)
        self.A = sk["A"]
        log("skewed")
        # ---- prefill: partial weight index (Section 4.3), query-only ranking on Q~ = Qcal A ----
        Qs = ig.ig_apply_skew(Qcal, self.A, ctx=ctx)
        self.idx_host = ig.ig_partial_index(Qs, None, w.H, w.ratio, ctx=ctx)
        self.r = self.idx_host.shape[1]
        self.desc = ig.IgDesc(B=w.B, H=w.H, d=w.d, r=self.r, N=w.N, N_cap=self.N_cap,
                              dtype=ig.IG_F32 if w.dtype == "f32" else ig.IG_F16,
                              scale=self.gain / math.sqrt(w.d), alpha=w.alpha,
                              rope=1 if w.rope else 0)
        self.idx = torch.from_numpy(self.idx_host).to(dev)
        W_in = Wq if w.rope else sk["Wq_s"]
        self.W_host = wl.quantise(W_in, w)
        Wd = torch.from_numpy(self.W_host).to(dev)
        self.wq = torch.empty(ig.ig_wq_bytes(self.desc), dtype=torch.uint8, device=dev)
        ctx.ig_wq_build(self.desc, Wd, self.idx, self.wq)
        self.A_p = self.pos = None
        if w.rope:
            A_p = np.stack([self.A[h][:, self.idx_host[h]] for h in range(w.H)]).astype(np.float32)
            self.A_p = torch.from_numpy(np.ascontiguousarray(A_p)).to(dev)
            self.pos = torch.full((w.B,), w.N, dtype=torch.int32, device=dev)
        self._Wd = Wd                      # weight the stand-in model uses for the layer's real query
        ctx.ig_reserve(self.desc)
        log("partial weight built")
        self._build_layers(host_layers, sets, log)

    def _build_layers(self, host_layers, sets, log):
        """Per-layer state: layer inputs, the layer's real query, KV pool, partial key cache."""
        ctx, w, dev, tdt = self.ctx, self.w, "cuda", self.tdt
        extra_tokens = self.N_cap - w.N
        Wq_model = self._Wd
        self.host_pool = w.pool == "host"
        self.n_pool = min(self.L, host_layers) if self.host_pool else self.L
        self.x, self.q, self.slab, self.K, self.V = [], [], [], [], []
        slab_bytes = ig.ig_slab_bytes(self.desc)
        for l in range(self.L):
            if l == 0:
                x = torch.from_numpy(wl.quantise(wl.attention_input(w, 0), w)).to(dev)
                xn = torch.from_numpy(wl.next_layer_input(w, x.float().cpu().numpy(), 0)).to(dev)
                Kn, Vn = wl.kv_cache(w, 0)          # keys are drawn directly in the skewed basis
                K = torch.from_numpy(wl.quantise(Kn, w))
                V = torch.from_numpy(wl.quantise(Vn, w))
                del Kn, Vn
                self.layer0_host = dict(x=x.cpu().numpy(), K=K.numpy(), V=V.numpy())
                K, V = K.to(dev), V.to(dev)
                if extra_tokens:
                    pad = torch.zeros((w.B, w.H, extra_tokens, w.d), dtype=K.dtype, device=dev)
                    K, V = torch.cat([K, pad], 2).contiguous(), torch.cat([V, pad], 2).contiguous()
            else:
                g = torch.Generator(device=dev).manual_seed(1000 * w.cfg + 7919 * l)
                x = torch.randn((w.B, w.D), generator=g, device=dev).to(tdt)
                xn = x.float() + 0.3 * torch.randn((w.B, w.D), generator=g, device=dev)
                K = torch.randn((w.B, w.H, self.N_cap, w.d), generator=g, device=dev, dtype=tdt)
                V = torch.randn((w.B, w.H, self.N_cap, w.d), generator=g, device=dev, dtype=tdt)
                gain_rows = torch.from_numpy(wl.key_row_gain(w, l)).to(dev).to(tdt)
                K[:, :, :w.N] *= gain_rows[:, None, :, None]
            # the layer's real (skewed) query: the stand-in model's projection of its own input
            qf = (xn.to(tdt) @ Wq_model).float().reshape(w.B, w.H, w.d)
            if w.rope:
                qh = ig.ig_rope_rows(qf.cpu().numpy(), np.full(w.B, w.N), ctx=ctx)
                qf = torch.from_numpy(ig.ig_apply_skew(qh.reshape(w.B, w.D), self.A, ctx=ctx)
                                      ).to(dev).reshape(w.B, w.H, w.d)
            q = qf.to(tdt).contiguous()
            slab = torch.empty(slab_bytes, dtype=torch.uint8, device=dev)
            ctx.ig_slab_build(self.desc, K, ig.IG_MEM_DEVICE, self.idx, slab)
            torch.cuda.synchronize()
            self.x.append(x)
            self.q.append(q)
            self.slab.append(slab)
            if l == 0:
                self.layer0_host["q"] = q.cpu().numpy()
            if self.host_pool:
                if l < self.n_pool:
                    Kh = torch.empty(K.shape, dtype=tdt, pin_memory=True)
                    Vh = torch.empty(V.shape, dtype=tdt, pin_memory=True)
                    Kh.copy_(K)
                    Vh.copy_(V)
                    self.K.append(Kh)
                    self.V.append(Vh)
                del K, V
            else:
                self.K.append(K)
                self.V.append(V)
        log("layers built")
        self.space = ig.IG_MEM_HOST_PINNED if self.host_pool else ig.IG_MEM_DEVICE
        BH = w.B * w.H
        self.stride = self.N_cap
        # result buffers; a host pool is pipelined over two sets (rehearsal of layer l+1 runs while the
        # rows of layer l are still crossing PCIe)
        self.n_sets = sets
        self.sets = []
        for _ in range(self.n_sets):
            self.sets.append(dict(
                sel_idx=torch.zeros((BH, self.stride), dtype=torch.int32, device=dev),
                sel_cnt=torch.zeros((BH,), dtype=torch.int32, device=dev),
                K_sel=torch.zeros((BH, self.stride, w.d), dtype=tdt, device=dev),
                V_sel=torch.zeros((BH, self.stride, w.d), dtype=tdt, device=dev)))
        self._use(0)
        self.out = torch.zeros((w.B, w.H, w.d), dtype=tdt, device=dev)
        self.side_ctx = ig.Context(0)              # the side stream gets its own context
        self.side_ctx.ig_reserve(self.desc)
        self.side = torch.cuda.Stream()

    def _use(self, i):
        st = self.sets[i % self.n_sets]
        self.sel_idx, self.sel_cnt, self.K_sel, self.V_sel = st["sel_idx"], st["sel_cnt"], st["K_sel"], st["V_sel"]

    # ---- hot path ----
    def speculate(self, l, scores=None):
        self.ctx.ig_speculate(self.desc, self.x[l], self.wq, None, self.A_p, self.pos, self.slab[l],
                              self.sel_idx, self.stride, self.sel_cnt, scores)

    def speculate_index_only(self, l, scores=None):
        """Rehearsal with the index-only partial weight (Section 6.2 "Memory Consumption"): the kept
        columns are read out of the model's full skewed query weight; no weight blob is used."""
        self.ctx.ig_speculate_indexed(self.desc, self.x[l], self._Wd, self.idx, None, self.slab[l],
                                      self.sel_idx, self.stride, self.sel_cnt, scores)

    def gather(self, l, stream=None):
        p = l % self.n_pool
        self.ctx.ig_gather_kv(self.desc, self.K[p], self.V[p], self.space, self.sel_idx, self.stride,
                              self.sel_cnt, self.K_sel, self.V_sel, stream)

    def attend(self, l):
        self.ctx.ig_sparse_attention(self.desc, self.q[l], self.K_sel, self.V_sel, self.sel_cnt,
                                     self.stride, None, None, self.out)

    def attend_indexed(self, l):
        p = l % self.n_pool
        self.ctx.ig_sparse_attention_indexed(self.desc, self.q[l], self.K[p], self.V[p], self.sel_idx,
                                             self.stride, self.sel_cnt, None, None, self.out)

    def gather_attend(self, l):
        p = l % self.n_pool
        self.ctx.ig_gather_attention(self.desc, self.q[l], self.K[p], self.V[p], self.sel_idx,
                                     self.stride, self.sel_cnt, self.K_sel, self.V_sel, None, None,
                                     self.out)

    def layer(self, l):
        """Rehearsal, prefetch and sparse attention of one layer on the current stream."""
        self.speculate(l)
        self.gather(l)
        self.attend(l)

    def step(self):
        """One decode step: every layer once (distinct slabs, so nothing is served from cache)."""
        for l in range(self.L):
            self.layer(l)

    def step_without_gather(self):
        """Main-stream work of a host-pool step alone: rehearsal + attention on whatever was fetched."""
        for l in range(self.L):
            self._use(l)
            self.speculate(l)
            self.attend(l)

    def collect_lists(self):
        """Every layer's own index lists, kept for step_gather_only (the pipelined step reuses two
        list buffers, which would leave only the last two layers' lists behind)."""
        self.layer_lists = []
        for l in range(self.L):
            self._use(l)
            self.speculate(l)
            self.layer_lists.append((self.sel_idx.clone(), self.sel_cnt.clone()))
        torch.cuda.synchronize()

    def step_gather_only(self):
        """Side-stream work of a host-pool step alone: the prefetch of every layer with that
        layer's own lists (collect_lists() first)."""
        for l in range(self.L):
            self._use(l)
            p = l % self.n_pool
            sel_idx, sel_cnt = self.layer_lists[l]
            self.side_ctx.ig_gather_kv(self.desc, self.K[p], self.V[p], self.space, sel_idx,
                                       self.stride, sel_cnt, self.K_sel, self.V_sel, self.side)

    def step_fused_attention(self):
        """Variant for an HBM-resident pool: the index lists are applied inside the attention."""
        for l in range(self.L):
            self.speculate(l)
            self.attend_indexed(l)

    def host_speculation_setup(self, slab_layers: int = 4):
        """Moves the partial key cache of `slab_layers` layers to host memory (later layers reuse
        them in turn) and allocates the pinned staging buffers of step_host_speculation."""
        w, BH = self.w, self.w.B * self.w.H
        n = min(self.L, slab_layers)
        self.slab_host = [self.slab[l].cpu().pin_memory() for l in range(n)]
        self.q_p = torch.empty((w.B, w.H, self.r), device="cuda")
        self.q_p_host = torch.empty((w.B, w.H, self.r), pin_memory=True)
        self.sel_idx_host = torch.zeros((BH, self.stride), dtype=torch.int32, pin_memory=True)
        self.sel_cnt_host = torch.zeros((BH,), dtype=torch.int32, pin_memory=True)

    def step_host_speculation(self, threads: int = 0, after_layer=None):
        """Decode step with the partial key cache in host memory and the speculation on the CPU
        (Section 6.2 "Memory Consumption"): per layer the GPU projects the partial query, the host
        fetches it, scans its copy of the partial key cache and builds the lists, the lists go back
        and the GPU prefetches and attends as usual."""
        for l in range(self.L):
            self.ctx.ig_project(self.desc, self.x[l], self.wq, None, self.A_p, self.pos, self.q_p)
            self.q_p_host.copy_(self.q_p, non_blocking=True)
            torch.cuda.current_stream().synchronize()
            rc = ig.lib().ig_speculate_host(self.ctx._h, ig.ctypes.byref(self.desc), self.q_p_host.data_ptr(),
                                            self.slab_host[l % len(self.slab_host)].data_ptr(),
                                            self.sel_idx_host.data_ptr(), self.stride,
                                            self.sel_cnt_host.data_ptr(), None, threads)
            if rc != ig.IG_OK:
                raise ig.IgError(rc, self.ctx.last_error())
            self.sel_idx.copy_(self.sel_idx_host, non_blocking=True)
            self.sel_cnt.copy_(self.sel_cnt_host, non_blocking=True)
            self.gather(l)
            self.attend(l)
            if after_layer is not None:
                torch.cuda.current_stream().synchronize()
                after_layer(l)

    def step_overlapped(self, after_layer=None):
        """Host-pool decode step (Fig. 3(d)): the rows of layer l are prefetched over PCIe on a side
        stream while the main stream already rehearses layer l+1 and attends layer l-1.
        after_layer(l), if given, is called right after layer l's attention has been enqueued and
        before its buffer set is released to the side stream (whatever it enqueues on the current
        stream sees that layer's lists, fetched rows and output)."""
        main = torch.cuda.current_stream()
        ev_spec = [None] * self.L
        ev_gath = [None] * self.L
        ev_attn = [None] * self.L
        for l in range(self.L + 1):
            if l < self.L:
                self._use(l)
                # the lists of this set are free: the attention that read them was enqueued earlier
                self.speculate(l)
                ev_spec[l] = torch.cuda.Event()
                ev_spec[l].record(main)
                self.side.wait_event(ev_spec[l])
                if l >= self.n_sets:
                    self.side.wait_event(ev_attn[l - self.n_sets])   # K_sel/V_sel set is free again
                p = l % self.n_pool
                self.side_ctx.ig_gather_kv(self.desc, self.K[p], self.V[p], self.space, self.sel_idx,
                                           self.stride, self.sel_cnt, self.K_sel, self.V_sel, self.side)
                ev_gath[l] = torch.cuda.Event()
                ev_gath[l].record(self.side)
            if l >= 1:
                self._use(l - 1)
                main.wait_event(ev_gath[l - 1])
                self.attend(l - 1)
                if after_layer is not None:
                    after_layer(l - 1)
                ev_attn[l - 1] = torch.cuda.Event()
                ev_attn[l - 1].record(main)

    def step_overlapped_native(self):
        """The same step issued by the library (ig_decode_step_overlapped): one call enqueues every
        layer's rehearsal, prefetch and attention on the two streams with the events between them.
        Every layer writes its own output row block (self.outs[l])."""
        if not hasattr(self, "_native_layers"):
            self.outs = [torch.zeros_like(self.out) for _ in range(self.L)]
            L_t = ig.IgLayerIO * self.L
            S_t = ig.IgBufferSet * self.n_sets
            self._native_layers = L_t(*[
                ig.IgLayerIO(x=self.x[l].data_ptr(), slab=self.slab[l].data_ptr(), q=self.q[l].data_ptr(),
                             Kpool=self.K[l % self.n_pool].data_ptr(), Vpool=self.V[l % self.n_pool].data_ptr(),
                             k_new=None, v_new=None, out=self.outs[l].data_ptr()) for l in range(self.L)])
            self._native_sets = S_t(*[
                ig.IgBufferSet(sel_idx=st["sel_idx"].data_ptr(), sel_cnt=st["sel_cnt"].data_ptr(),
                               K_sel=st["K_sel"].data_ptr(), V_sel=st["V_sel"].data_ptr()) for st in self.sets])
        self.ctx.ig_decode_step_overlapped(self.desc, self._native_layers, self.wq, None, self.A_p, self.pos,
                                           self.space, self._native_sets, self.stride,
                                           torch.cuda.current_stream(), self.side)

    def step_one_pass(self):
        """HBM-pool decode step with prefetch and attention in one pass over the pool."""
        for l in range(self.L):
            self.speculate(l)
            self.gather_attend(l)

    def step_joint(self):
        """HBM-pool decode step on one stream with ig_layer_step: after the first layer's rehearsal,
        every call issues the next layer's projection and then ONE launch that holds the next
        layer's scan / threshold / lists and this layer's prefetch + attention (Fig. 3(d): the next
        layer is speculated while the current one computes).  The index lists and fetched rows are
        double-buffered."""
        self._use(0)
        self.speculate(0)
        for l in range(self.L):
            cur, nxt = self.sets[l % self.n_sets], self.sets[(l + 1) % self.n_sets]
            p = l % self.n_pool
            if l + 1 < self.L:
                self.ctx.ig_layer_step(self.desc, self.x[l + 1], self.wq, None, self.A_p, self.pos,
                                       self.slab[l + 1], nxt["sel_idx"], nxt["sel_cnt"], self.q[l],
                                       self.K[p], self.V[p], cur["sel_idx"], cur["sel_cnt"], self.stride,
                                       cur["K_sel"], cur["V_sel"], None, None, self.out)
            else:
                self.ctx.ig_gather_attention(self.desc, self.q[l], self.K[p], self.V[p], cur["sel_idx"],
                                             self.stride, cur["sel_cnt"], cur["K_sel"], cur["V_sel"],
                                             None, None, self.out)
        self._use(self.L - 1)

    def step_index_only(self):
        """step_one_pass() with the index-only partial weight (host pool: the rehearsals only, the
        prefetch over PCIe does not depend on where the weight columns come from)."""
        for l in range(self.L):
            self.speculate_index_only(l)
            if not self.host_pool:
                self.gather_attend(l)

    def step_equalized(self, max_frac=0.2):
        """The paper's batched variant (Section 4.3, closing sentences): every head of a sequence
        fetches the same number of tokens.  Rehearsal with equalised lists in one call (for the
        shapes that allow it the scan kernel selects each head's top n itself), then prefetch and
        attention over the equalised lists (HBM pool: in one pass)."""
        for l in range(self.L):
            self.ctx.ig_speculate_equalized(self.desc, self.x[l], self.wq, None, self.A_p, self.pos,
                                            self.slab[l], max_frac, self.sel_idx, self.stride, self.sel_cnt)
            if self.host_pool:
                self.gather(l)
                self.attend(l)
            else:
                self.gather_attend(l)

    def step_equalized_two_calls(self, max_frac=0.2):
        """The same through ig_speculate (scores kept) and ig_equalize_heads."""
        w = self.w
        if not hasattr(self, "scores"):
            self.scores = torch.zeros((w.B, w.H, w.N), device="cuda")
            self.thr_idx = torch.zeros_like(self.sets[0]["sel_idx"])
            self.thr_cnt = torch.zeros_like(self.sets[0]["sel_cnt"])
        for l in range(self.L):
            self.ctx.ig_speculate(self.desc, self.x[l], self.wq, None, self.A_p, self.pos, self.slab[l],
                                  self.thr_idx, self.stride, self.thr_cnt, self.scores)
            self.ctx.ig_equalize_heads(self.desc, self.scores, self.thr_cnt, max_frac, self.sel_idx,
                                       self.stride, self.sel_cnt)
            if self.host_pool:
                self.gather(l)
                self.attend(l)
            else:
                self.gather_attend(l)

    def step_two_stream(self, one_pass=True):
        """HBM-pool decode step with the rehearsal on a side stream (Fig. 3(d): the next layer is
        speculated while the current one computes): the side stream runs ig_speculate of layer l+1
        while the current stream gathers and attends layer l.  The index lists are double-buffered.
        Works eagerly and under stream capture (the side stream forks from and joins the current
        stream through events)."""
        main = torch.cuda.current_stream()
        side = self.side
        side.wait_stream(main)
        ev_attn = [None] * self.L
        for l in range(self.L):
            self._use(l)
            if l >= self.n_sets:
                side.wait_event(ev_attn[l - self.n_sets])    # this set's lists are free again
            self.side_ctx.ig_speculate(self.desc, self.x[l], self.wq, None, self.A_p, self.pos,
                                       self.slab[l], self.sel_idx, self.stride, self.sel_cnt, None, side)
            ev = torch.cuda.Event()
            ev.record(side)
            main.wait_event(ev)
            if one_pass:
                self.gather_attend(l)
            else:
                self.gather(l)
                self.attend(l)
            ev_attn[l] = torch.cuda.Event()
            ev_attn[l].record(main)
        main.wait_stream(side)

    def decode(self, steps: int, dense_first_layer: bool = True, after_layer=None):
        """`steps` decode steps over all layers with a growing cache (Section 2.1, Section 4.3):
        per layer the rehearsal, prefetch and attention over the cached tokens plus the token being
        decoded, then that token's key / value are appended to the layer's pool and slab.  The first
        layer attends every token (speculation starts at the second layer, Section 4.3).  Needs
        extra_tokens >= steps.  Single stream; the synthetic new-token rows are fixed tensors.
        after_layer(step, l), if given, is called after a layer's attention has been enqueued and
        before its append."""
        w = self.w
        assert self.w.N + steps <= self.N_cap, "construct with extra_tokens >= steps"
        if not hasattr(self, "k_new"):
            g = torch.Generator(device="cuda").manual_seed(4242 + w.cfg)
            self.k_new = torch.randn((w.B, w.H, w.d), generator=g, device="cuda").to(self.tdt)
            self.v_new = torch.randn((w.B, w.H, w.d), generator=g, device="cuda").to(self.tdt)
            self.desc_dense = ig.IgDesc(B=w.B, H=w.H, d=w.d, r=self.r, N=w.N, N_cap=self.N_cap,
                                        dtype=self.desc.dtype, scale=self.desc.scale,
                                        alpha=float("inf"), rope=self.desc.rope)
        self._use(0)
        n0 = self.desc.N
        for s_ in range(steps):
            for l in range(self.L):
                d = self.desc_dense if (dense_first_layer and l == 0) else self.desc
                d.N = n0 + s_
                p = l % self.n_pool
                self.ctx.ig_speculate(d, self.x[l], self.wq, None, self.A_p, self.pos, self.slab[l],
                                      self.sel_idx, self.stride, self.sel_cnt, None)
                if self.host_pool:
                    self.ctx.ig_gather_kv(d, self.K[p], self.V[p], self.space, self.sel_idx, self.stride,
                                          self.sel_cnt, self.K_sel, self.V_sel)
                    self.ctx.ig_sparse_attention(d, self.q[l], self.K_sel, self.V_sel, self.sel_cnt,
                                                 self.stride, self.k_new, self.v_new, self.out)
                else:
                    self.ctx.ig_gather_attention(d, self.q[l], self.K[p], self.V[p], self.sel_idx,
                                                 self.stride, self.sel_cnt, self.K_sel, self.V_sel,
                                                 self.k_new, self.v_new, self.out)
                if after_layer is not None:
                    after_layer(s_, l)
                self.ctx.ig_append_token(d, self.k_new, self.v_new, self.idx, self.slab[l], self.K[p],
                                         self.V[p], self.space)
        self.desc.N = n0
        self.desc_dense.N = n0

    def gathered_bytes(self) -> int:
        """Bytes the prefetch of the layer whose lists are current moves (K and V rows)."""
        w = self.w
        return int(self.sel_cnt.sum().item()) * 2 * w.d * (4 if w.dtype == "f32" else 2)

    def scan_bytes(self) -> int:
        """Algorithmic bytes of one partial-K scan: 2*B*H*N*r (elements actually needed)."""
        w = self.w
        return w.B * w.H * w.N * self.r * (4 if w.dtype == "f32" else 2)
