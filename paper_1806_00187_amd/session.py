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
    def __init__(self, model, weights, max_sentences=1024, max_len=256, act_dropout=0.0, label_smoothing=0.1, ln_eps=1e-5,
                 seed=0, pad_id=1, device="cuda:0", optimizer=True):
        """model: dict(enc_layers, dec_layers, d_model, n_heads, d_ff, vocab, dropout);
        weights: dict name -> float16 numpy array (initial fp16 weights = initial master values)."""
        self.device = torch.device(device)
        self.model = dict(model)
        self.ctx = nmt.nmt_create(enc_layers=model["enc_layers"], dec_layers=model["dec_layers"], d_model=model["d_model"],
                                  n_heads=model["n_heads"], d_ff=model["d_ff"], vocab=model["vocab"], pad_id=pad_id,
                                  dropout=model.get("dropout", 0.0), act_dropout=act_dropout, label_smoothing=label_smoothing,
                                  ln_eps=ln_eps, seed=seed, max_sentences=max_sentences, max_len=max_len)
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
        self.g16 = torch.zeros(self.P, dtype=torch.float16, device=self.device)
        if optimizer:
            self.master = self.w16.float()
            self.acc = torch.zeros(self.P, dtype=torch.float32, device=self.device)
            self.m = torch.zeros_like(self.acc)
            self.v = torch.zeros_like(self.acc)
        else:
            self.master = self.acc = self.m = self.v = None
        self.workspace = None
        self.loss_sum = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.ntok = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.flag = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._bind()

    def _bind(self):
        nmt.nmt_bind(self.ctx, self.w16, self.g16, self.master, self.acc, self.m, self.v, self.workspace)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.device)
            nmt.nmt_destroy(self.ctx)
            self.ctx = None

    def reserve(self, B, S, T):
        need = nmt.nmt_workspace_bytes(self.ctx, B, S, T)
        if self.workspace is None or self.workspace.numel() < need:
            torch.cuda.synchronize(self.device)
            self.workspace = None
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
            self._bind()

    def to_device(self, batch):
        """numpy micro-batch -> dict of int32 device tensors (+ optional uint32 sentence ids)."""
        out = {k: torch.from_numpy(np.ascontiguousarray(batch[k], dtype=np.int32)).to(self.device) for k in ("src", "tgt_in", "tgt_out")}
        if batch.get("sent_uid") is not None:
            out["sent_uid"] = torch.from_numpy(np.ascontiguousarray(batch["sent_uid"]).astype(np.int64).astype(np.int32)).to(self.device)
        return out

    # ---- the five calls ----
    def forward_loss(self, dbatch, loss_scale, step, micro=0, training=True):
        B, S = dbatch["src"].shape
        self.reserve(B, S, dbatch["tgt_in"].shape[1])
        nmt.nmt_forward_loss(self.ctx, dbatch["src"], dbatch["tgt_in"], dbatch["tgt_out"], loss_scale, step, micro, self.loss_sum,
                             self.ntok, sent_uid=dbatch.get("sent_uid"), training=training)

    def backward(self):
        nmt.nmt_backward(self.ctx)

    def accumulate(self, first):
        nmt.nmt_accumulate(self.ctx, first)

    def check_overflow(self, inv_scale):
        nmt.nmt_check_overflow(self.ctx, inv_scale, self.flag)

    def adam_step(self, lr, t, betas=(0.9, 0.98), eps=1e-8):
        nmt.nmt_adam_step(self.ctx, lr, betas[0], betas[1], eps, t, self.flag)

    # ---- one weight update from k micro-batches ----
    def update(self, dbatches, loss_scale, lr, t, step=None, betas=(0.9, 0.98), eps=1e-8):
        """Returns (loss_sum, n_tok, overflow flag).  Synchronises once, to read the three scalars."""
        step = t if step is None else step
        loss_tot = torch.zeros(1, dtype=torch.float32, device=self.device)
        ntok_tot = torch.zeros(1, dtype=torch.int32, device=self.device)
        for j, db in enumerate(dbatches):
            self.forward_loss(db, loss_scale, step, j)
            self.backward()
            self.accumulate(j == 0)
            loss_tot += self.loss_sum
            ntok_tot += self.ntok
        n_tok = int(ntok_tot.item())
        self.check_overflow(1.0 / (loss_scale * max(n_tok, 1)))
        self.adam_step(lr, t, betas, eps)
        return float(loss_tot.item()), n_tok, int(self.flag.item())

    # ---- views for tests ----
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

    def step(self, dbatches, scale_override=None):
        scale = self.scale if scale_override is None else scale_override
        loss, ntok, flag = self.s.update(dbatches, scale, self.lr(), self.t)
        self.scale, self.clean = nmt.nmt_scaler_update(self.scale, self.clean, flag, self.window)
        if not flag:
            self.t += 1          # a skipped update advances neither Adam's step nor the schedule
        return loss, ntok, flag
