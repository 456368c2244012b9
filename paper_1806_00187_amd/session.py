"""Device-memory plumbing around the C ABI: a Session owns the torch tensors the library works on
(fp16 weights and gradients, fp32 master weights / accumulator / Adam moments, workspace) and
strings the five entry points together into one weight update.  Every arithmetic step runs in
the library's kernels; the only host logic here is the scalar loss-scale / learning-rate
bookkeeping, which itself calls the library's helpers."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as nmt


class Session:
    """n_pipes > 1 keeps that many sub-batches in flight: each pipe has its own library context (same
    weights and optimizer buffers, own fp16 gradient buffer and workspace) and its own HIP stream, so
    the forward pass of one sub-batch overlaps the backward pass of the previous one.  Accumulation
    into the shared fp32 buffer is chained with events in sub-batch order, which keeps the sum
    deterministic.  How well the pipes overlap depends on how the runtime spreads the process's streams over its few
    hardware queues, which a caller does not control: the same sixteen-sub-batch update of the big model measured
    107 ms with four pipes in a process that had no other stream of its own, and 134-137 ms when a stream created
    earlier (another session's second stream; it need not carry any work) was still alive.  So the first update of a
    session with several pipes times a few sets of streams on its own sub-batches and keeps the fastest
    (choose_streams; auto_streams=False keeps the streams as created)."""

    def __init__(self, model, weights, max_sentences=1024, max_len=256, act_dropout=0.0, label_smoothing=0.1, ln_eps=1e-5,
                 seed=0, pad_id=1, device="cuda:0", optimizer=True, n_pipes=1, auto_streams=True):
        """model: dict(enc_layers, dec_layers, d_model, n_heads, d_ff, vocab, dropout);
        weights: dict name -> float16 numpy array (initial fp16 weights = initial master values)."""
        self.device = torch.device(device)
        self.model = dict(model)
        self.n_pipes = n_pipes
        cfg = dict(enc_layers=model["enc_layers"], dec_layers=model["dec_layers"], d_model=model["d_model"],
                   n_heads=model["n_heads"], d_ff=model["d_ff"], vocab=model["vocab"], pad_id=pad_id,
                   dropout=model.get("dropout", 0.0), act_dropout=act_dropout, label_smoothing=label_smoothing,
                   ln_eps=ln_eps, seed=seed, max_sentences=max_sentences, max_len=max_len)
        self.ctxs = [nmt.nmt_create(**cfg) for _ in range(n_pipes)]
        self.ctx = self.ctxs[0]
        self.P = nmt.nmt_param_count(self.ctx)
        self.layout = {}
        for i in range(nmt.nmt_param_tensors(self.ctx)):
            name, off, rows, cols = nmt.nmt_param_info(self.ctx, i)
            self.layout[name] = (off, rows, cols)
        flat = np.zeros(self.P, dtype=np.float16)
        for name, (off, rows, cols) in self.layout.items():
            w = np.asarray(weights[name], dtype=np.float16)
            assert w.size == rows * cols, name
            flat[off:off + rows * cols] = w.reshape(-1)
        self.w16 = torch.from_numpy(flat).to(self.device)
        self.g16s = [torch.zeros(self.P, dtype=torch.float16, device=self.device) for _ in range(n_pipes)]
        self.g16 = self.g16s[0]
        if optimizer:
            self.master = self.w16.float()
            self.acc = torch.zeros(self.P, dtype=torch.float32, device=self.device)
            self.m = torch.zeros_like(self.acc)
            self.v = torch.zeros_like(self.acc)
        else:
            self.master = self.acc = self.m = self.v = None
        self.workspaces = [None] * n_pipes
        self.loss_sums = [torch.zeros(1, dtype=torch.float32, device=self.device) for _ in range(n_pipes)]
        self.ntoks = [torch.zeros(1, dtype=torch.int32, device=self.device) for _ in range(n_pipes)]
        self.loss_sum, self.ntok = self.loss_sums[0], self.ntoks[0]
        self.flag = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.loss_tot = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.ntok_tot = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.streams = [torch.cuda.Stream(device=self.device) for _ in range(n_pipes)] if n_pipes > 1 else [None]
        # with several pipes, the first update tries a few sets of streams and keeps the best (choose_streams)
        self._streams_chosen = n_pipes == 1 or not auto_streams
        for p in range(n_pipes):
            self._bind(p)

    def _bind(self, pipe=0):
        nmt.nmt_bind(self.ctxs[pipe], self.w16, self.g16s[pipe], self.master, self.acc, self.m, self.v, self.workspaces[pipe])

    @property
    def workspace(self):
        return self.workspaces[0]

    def close(self):
        if self.ctxs:
            torch.cuda.synchronize(self.device)
            for c in self.ctxs:
                nmt.nmt_destroy(c)
            self.ctxs, self.ctx = [], None

    def reserve(self, B, S=None, T=None):
        """Workspace for one (B, S, T) batch, or for a group given as a list of (B, S, T, micro)."""
        self._reserve_bytes(nmt.nmt_workspace_bytes_group(self.ctx, B) if S is None else nmt.nmt_workspace_bytes(self.ctx, B, S, T))

    def _reserve_bytes(self, need):
        for p in range(self.n_pipes):
            if self.workspaces[p] is None or self.workspaces[p].numel() < need:
                torch.cuda.synchronize(self.device)
                self.workspaces[p] = None
                self.workspaces[p] = torch.empty(need, dtype=torch.uint8, device=self.device)
                self._bind(p)

    def to_device(self, batch):
        """numpy micro-batch -> dict of int32 device tensors (+ optional uint32 sentence ids)."""
        out = {k: torch.from_numpy(np.ascontiguousarray(batch[k], dtype=np.int32)).to(self.device) for k in ("src", "tgt_in", "tgt_out")}
        if batch.get("sent_uid") is not None:
            out["sent_uid"] = torch.from_numpy(np.ascontiguousarray(batch["sent_uid"]).astype(np.int64).astype(np.int32)).to(self.device)
        return out

    @staticmethod
    def group(dbatches, size):
        """Stacks consecutive device sub-batches into groups of `size` that one forward / backward pass
        processes together; sub-batch j keeps micro index j (its dropout streams)."""
        out = []
        for g0 in range(0, len(dbatches), size):
            chunk = dbatches[g0:g0 + size]
            grp = {"segs": [(b["src"].shape[0], b["src"].shape[1], b["tgt_in"].shape[1], g0 + i) for i, b in enumerate(chunk)]}
            for k in ("src", "tgt_in", "tgt_out"):
                grp[k] = torch.cat([b[k].reshape(-1) for b in chunk])
            uids = [b.get("sent_uid") for b in chunk]
            assert all(u is None for u in uids) or all(u is not None for u in uids)
            grp["sent_uid"] = None if uids[0] is None else torch.cat(uids)
            out.append(grp)
        return out

    def pack(self, batches, size=None, pad_id=1):
        """Host sub-batches (numpy, right-padded) -> packed passes: the sentences of `size` consecutive sub-batches (all if
        None) back to back without padding, plus the per-sentence table (src_len, tgt_len, uid, micro).  Sub-batch j keeps micro
        index j; a sentence's uid is its `sent_uid` entry or its index within its sub-batch."""
        size = len(batches) if size is None else size
        out = []
        for g0 in range(0, len(batches), size):
            sent, src, tin, tout = [], [], [], []
            for j in range(g0, min(len(batches), g0 + size)):
                b = batches[j]
                uid = b.get("sent_uid")
                for i in range(b["src"].shape[0]):
                    ls, lt = int((b["src"][i] != pad_id).sum()), int((b["tgt_out"][i] != pad_id).sum())
                    assert ls >= 1 and lt >= 1 and (b["src"][i, ls:] == pad_id).all() and (b["tgt_out"][i, lt:] == pad_id).all()
                    sent.append((ls, lt, int(uid[i]) if uid is not None else i, j))
                    src.append(b["src"][i, :ls])
                    tin.append(b["tgt_in"][i, :lt])
                    tout.append(b["tgt_out"][i, :lt])
            tab = np.asarray(sent, dtype=np.int64)
            dev = lambda parts: torch.from_numpy(np.ascontiguousarray(np.concatenate(parts), dtype=np.int32)).to(self.device)
            out.append({"packed": torch.from_numpy(tab.astype(np.uint32).view(np.int32).reshape(-1, 4).copy()).to(self.device),
                        "n_src": int(tab[:, 0].sum()), "n_tgt": int(tab[:, 1].sum()), "max_src": int(tab[:, 0].max()),
                        "max_tgt": int(tab[:, 1].max()), "src": dev(src), "tgt_in": dev(tin), "tgt_out": dev(tout)})
        return out

    def _reserve_for(self, dbatch):
        """Workspace (of every pipe) large enough for this sub-batch, group or packed pass; nothing happens if it already is."""
        if "packed" in dbatch:
            self._reserve_bytes(nmt.nmt_workspace_bytes_packed(self.ctx, dbatch["packed"].shape[0], dbatch["n_src"], dbatch["n_tgt"]))
        elif "segs" in dbatch:
            self.reserve(dbatch["segs"])
        else:
            self.reserve(dbatch["src"].shape[0], dbatch["src"].shape[1], dbatch["tgt_in"].shape[1])

    # ---- the five calls ----
    def forward_loss(self, dbatch, loss_scale, step, micro=0, training=True, pipe=0):
        """dbatch: one device sub-batch (2-D id tensors), a group made by Session.group or a packed pass made by Session.pack
        (for the last two `micro` is unused)."""
        self._reserve_for(dbatch)
        if "packed" in dbatch:
            nmt.nmt_forward_loss_packed(self.ctxs[pipe], dbatch["packed"], dbatch["n_src"], dbatch["n_tgt"], dbatch["max_src"],
                                        dbatch["max_tgt"], dbatch["src"], dbatch["tgt_in"], dbatch["tgt_out"], loss_scale, step,
                                        self.loss_sums[pipe], self.ntoks[pipe], training=training)
            return
        if "segs" in dbatch:
            nmt.nmt_forward_loss_group(self.ctxs[pipe], dbatch["segs"], dbatch["src"], dbatch["tgt_in"], dbatch["tgt_out"], loss_scale,
                                       step, self.loss_sums[pipe], self.ntoks[pipe], sent_uid=dbatch.get("sent_uid"), training=training)
            return
        nmt.nmt_forward_loss(self.ctxs[pipe], dbatch["src"], dbatch["tgt_in"], dbatch["tgt_out"], loss_scale, step, micro,
                             self.loss_sums[pipe], self.ntoks[pipe], sent_uid=dbatch.get("sent_uid"), training=training)

    def grad_scale(self, pipe=0):
        """Power-of-two factor the last forward call's pass applies to what it writes to g16."""
        return nmt.nmt_grad_scale(self.ctxs[pipe])

    def backward(self, pipe=0):
        nmt.nmt_backward(self.ctxs[pipe])

    def accumulate(self, first, pipe=0):
        nmt.nmt_accumulate(self.ctxs[pipe], first)

    def check_overflow(self, inv_scale):
        nmt.nmt_check_overflow(self.ctx, inv_scale, self.flag)

    def adam_step(self, lr, t, betas=(0.9, 0.98), eps=1e-8):
        nmt.nmt_adam_step(self.ctx, lr, betas[0], betas[1], eps, t, self.flag)

    # ---- one weight update from k micro-batches ----
    def update(self, dbatches, loss_scale, lr, t, step=None, betas=(0.9, 0.98), eps=1e-8, n_tok=None):
        """dbatches: device sub-batches (sub-batch j gets micro index j) or groups made by Session.group.
        Returns (loss_sum, n_tok, overflow flag).  n_tok (the number of non-pad target tokens of the
        whole update) is known to whoever built the batches; if it is not passed it is read back from
        the device, which costs one more synchronisation."""
        step = t if step is None else step
        main = torch.cuda.current_stream(self.device)
        if self.n_pipes == 1:
            for j, db in enumerate(dbatches):
                self.forward_loss(db, loss_scale, step, j)
                self.backward()
                self.accumulate(j == 0)
                nmt.nmt_accumulate_loss(self.ctx, j == 0, self.loss_tot, self.ntok_tot)
        else:
            if not self._streams_chosen:
                self.choose_streams(dbatches, loss_scale, tries=4)
            self._update_pipes(dbatches, loss_scale, step, main)
        if n_tok is None:
            n_tok = int(self.ntok_tot.item())
        self.check_overflow(1.0 / (loss_scale * max(n_tok, 1)))
        self.adam_step(lr, t, betas, eps)
        return float(self.loss_tot.item()), n_tok, int(self.flag.item())

    def _update_pipes(self, dbatches, loss_scale, step, main):
        """Sub-batch j goes through pipe j % n_pipes; accumulation is chained with events in sub-batch order.  One host
        thread enqueues the sub-batches whole, one after the other: the pipes then run staggered (the forward pass of one
        beside the backward pass of another), which measured a quarter faster than pipes that start together, whether
        those are fed by a thread each or forward passes first."""
        for db in dbatches:
            self._reserve_for(db)
        start = torch.cuda.Event()
        start.record(main)
        # The products of the pipes run side by side: each takes large tiles as if it had its share of the chip, and
        # each pipe's weight gradients stay on its own stream (the pipes already fill the hardware queues).
        before = {k: nmt.tuning_value(k, d) for k, d in (("gemm_share", 1), ("one_stream", 0))}
        nmt.nmt_tuning("gemm_share", self.n_pipes)
        nmt.nmt_tuning("one_stream", 1)
        try:
            prev = None
            for j, db in enumerate(dbatches):
                p = j % self.n_pipes
                s = self.streams[p]
                if j < self.n_pipes:
                    s.wait_event(start)            # the weights of this update are in place
                with torch.cuda.stream(s):
                    self.forward_loss(db, loss_scale, step, j, pipe=p)
                    self.backward(pipe=p)
                    if prev is not None:
                        s.wait_event(prev)         # accumulate in sub-batch order
                    self.accumulate(j == 0, pipe=p)
                    nmt.nmt_accumulate_loss(self.ctxs[p], j == 0, self.loss_tot, self.ntok_tot)
                    prev = torch.cuda.Event()
                    prev.record(s)
        finally:
            for k, v in before.items():
                nmt.nmt_tuning(k, v)
        main.wait_event(prev)

    def choose_streams(self, dbatches, loss_scale=1.0, tries=6, log=None):
        """Picks the pipes' streams by measurement.  How well the pipes overlap depends on which hardware queues the
        runtime has put their streams on (see the class note), and nothing but a run tells: up to `tries` sets of
        streams each carry the forward + backward + accumulate part of one update over `dbatches` twice (weights and
        optimizer state are not touched; the gradient buffers and the accumulator are overwritten, as they are by
        the next update anyway), and the set whose second run was fastest is kept.  Returns its time in ms."""
        self._streams_chosen = True
        if self.n_pipes == 1:
            return None
        main = torch.cuda.current_stream(self.device)
        best = None
        for _ in range(tries):
            cand = [torch.cuda.Stream(device=self.device) for _ in range(self.n_pipes)]
            self.streams = cand
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for rep in range(2):
                torch.cuda.synchronize(self.device)
                t0.record(main)
                self._update_pipes(dbatches, loss_scale, 0, main)
                t1.record(main)
                torch.cuda.synchronize(self.device)
            ms = t0.elapsed_time(t1)
            if log:
                log(f"[session] stream set {[hex(s.cuda_stream) for s in cand]}: {ms:.1f} ms")
            if best is None or ms < best[0]:
                best = (ms, cand)
        self.streams = best[1]
        return best[0]

    # ---- views for tests ----
    def activation(self, name, pipe=0):
        """A saved fp16 activation of the last forward pass as a view into the workspace tensor."""
        ptr, rows, cols = nmt.nmt_debug_activation(self.ctxs[pipe], name)
        ws = self.workspaces[pipe]
        off = ptr - ws.data_ptr()
        assert 0 <= off and off + rows * cols * 2 <= ws.numel()
        return ws[off:off + rows * cols * 2].view(torch.float16).reshape(rows, cols)

    def tensor(self, flat, name):
        off, rows, cols = self.layout[name]
        return flat[off:off + rows * cols].reshape(rows, cols) if rows > 1 else flat[off:off + cols]

    def named(self, flat):
        host = flat.detach().cpu().numpy()
        return {name: self.tensor(host, name) for name in self.layout}


class Trainer:
    """Dynamic loss scaling and the learning-rate schedule around Session.update (scalars only)."""

    def __init__(self, session, peak_lr=5e-4, warmup=4000, init_scale=128.0, window=2000, constant_lr=False):
        self.s, self.peak_lr, self.warmup, self.window, self.constant_lr = session, peak_lr, warmup, window, constant_lr
        self.scale, self.clean, self.t = float(init_scale), 0, 1

    def lr(self):
        return self.peak_lr if self.constant_lr else nmt.nmt_lr_schedule(self.t, self.peak_lr, self.warmup)

    def step(self, dbatches, scale_override=None, n_tok=None):
        scale = self.scale if scale_override is None else scale_override
        loss, ntok, flag = self.s.update(dbatches, scale, self.lr(), self.t, n_tok=n_tok)
        self.scale, self.clean = nmt.nmt_scaler_update(self.scale, self.clean, flag, self.window)
        if not flag:
            self.t += 1          # a skipped update advances neither Adam's step nor the schedule
        return loss, ntok, flag
