"""Sub-batch construction (host logic; section "Analysis of Stragglers", the paragraph on sub-batches
that take about the same time to process).  Two rules over a population of sentence pairs sorted by length:

* token budget: as many sentences as fit B * max(S, T) <= N (the baseline rule);
* time balance: a table estimates the processing time of a sub-batch from its number of sentences
  and its longest source and target sentence; every sub-batch is grown, sentence by sentence, until
  the estimate reaches a fixed target (e.g. the 90th percentile of the token-budget sub-batches), so
  that workers which each process one sub-batch per step finish together.

The table is fitted to times measured with the library itself (`measure`), on whatever GPU it runs."""
from __future__ import annotations

import numpy as np


def _features(B, S, T):
    B, S, T = (np.asarray(v, dtype=np.float64) for v in (B, S, T))
    # a launch-bound floor, the row-wise work (projections, FFN, vocabulary) and the attention squares
    return np.stack([np.ones_like(B), B, B * S, B * T, B * S * S, B * T * T, B * S * T], axis=-1)


class TimeTable:
    """time(B, S, T) of one sub-batch, a non-negative least-squares fit over measured samples."""

    def __init__(self, samples):
        """samples: iterable of (B, S, T, seconds)."""
        arr = np.asarray(list(samples), dtype=np.float64)
        assert arr.ndim == 2 and arr.shape[1] == 4 and len(arr) >= 7, "need at least 7 (B, S, T, time) samples"
        from scipy.optimize import nnls
        X = _features(arr[:, 0], arr[:, 1], arr[:, 2])
        self.scale = X.max(axis=0)
        self.coef, _ = nnls(X / self.scale, arr[:, 3])
        self.samples = arr

    def __call__(self, B, S, T):
        return _features(B, S, T) / self.scale @ self.coef

    def max_rel_error(self):
        est = self(self.samples[:, 0], self.samples[:, 1], self.samples[:, 2])
        return float(np.max(np.abs(est - self.samples[:, 3]) / self.samples[:, 3]))


def sort_by_length(src_len, tgt_len):
    """Sentences of similar length next to each other: by target length, then source length."""
    return np.lexsort((np.asarray(src_len), np.asarray(tgt_len)))


def token_budget_batches(src_len, tgt_len, max_tokens):
    """Index arrays of sub-batches with B * max(S, T) <= max_tokens over the length-sorted population."""
    order = sort_by_length(src_len, tgt_len)
    out, cur, cur_max = [], [], 0
    for i in order:
        m = max(cur_max, int(src_len[i]), int(tgt_len[i]))
        if cur and (len(cur) + 1) * m > max_tokens:
            out.append(np.array(cur))
            cur, m = [], max(int(src_len[i]), int(tgt_len[i]))
        cur.append(i)
        cur_max = m
    if cur:
        out.append(np.array(cur))
    return out


def shape_of(idx, src_len, tgt_len):
    return len(idx), int(np.max(src_len[idx])), int(np.max(tgt_len[idx]))


def time_balanced_batches(src_len, tgt_len, table, target, max_sentences=None, max_tokens=None):
    """Sub-batches over the length-sorted population, each grown until one more sentence would push the
    table's estimate above `target` (or past the optional caps).  A sentence that alone exceeds the
    target still forms a sub-batch of its own."""
    order = sort_by_length(src_len, tgt_len)
    out, cur, S, T = [], [], 0, 0
    for i in order:
        s, t = max(S, int(src_len[i])), max(T, int(tgt_len[i]))
        b = len(cur) + 1
        over = float(table(b, s, t)) > target
        over = over or (max_sentences is not None and b > max_sentences)
        over = over or (max_tokens is not None and b * max(s, t) > max_tokens)
        if cur and over:
            out.append(np.array(cur))
            cur, s, t = [], int(src_len[i]), int(tgt_len[i])
        cur.append(i)
        S, T = s, t
    if cur:
        out.append(np.array(cur))
    return out


def target_time(batches, src_len, tgt_len, table, quantile=0.9):
    """The fixed target: a quantile (the 90th percentile by default) of the estimated times of a reference
    set of sub-batches."""
    est = [float(table(*shape_of(b, src_len, tgt_len))) for b in batches]
    return float(np.quantile(est, quantile))


def measure(session, shapes, vocab, loss_scale=1.0, reps=3, seed=0):
    """Seconds of forward + backward + accumulate of one sub-batch per (B, S, T) shape, measured with HIP
    events through `session` (full-length sentences, random ids)."""
    import torch
    rng = np.random.default_rng(seed)
    out = []
    for (B, S, T) in shapes:
        batch = {"src": rng.integers(4, vocab, size=(B, S)), "tgt_in": rng.integers(4, vocab, size=(B, T)),
                 "tgt_out": rng.integers(4, vocab, size=(B, T))}
        db = session.to_device(batch)

        def step():
            session.forward_loss(db, loss_scale, 1, 0)
            session.backward()
            session.accumulate(True)

        step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            step()
        e1.record()
        torch.cuda.synchronize()
        out.append((B, S, T, e0.elapsed_time(e1) * 1e-3 / reps))
    return out
