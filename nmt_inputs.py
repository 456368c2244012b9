"""Seeded synthetic inputs for the NMT training-step tests and benchmark.

Holds none of the method's arithmetic: only model shapes, random weight initialisation,
sentence-length / token-id sampling and token-budget batching.  Both the CPU oracle's tests
and the GPU path's tests draw their inputs from here so that they see identical data.

The length and token statistics stand in for the paper's WMT sub-batches (sub-batches of
similar-length sentences holding at most N tokens; 32K / 40K joint vocabularies), which are
not available offline.
"""
from __future__ import annotations

import numpy as np

PAD, BOS = 1, 2

# name -> model hyper-parameters (workload descriptions of the five benchmark configurations)
MODELS = {
    "tiny": dict(enc_layers=2, dec_layers=2, d_model=64, n_heads=4, d_ff=256, vocab=1000, dropout=0.1),
    "base": dict(enc_layers=6, dec_layers=6, d_model=512, n_heads=8, d_ff=2048, vocab=32768, dropout=0.1),
    "big": dict(enc_layers=6, dec_layers=6, d_model=1024, n_heads=16, d_ff=4096, vocab=32768, dropout=0.3),
    "big40k": dict(enc_layers=6, dec_layers=6, d_model=1024, n_heads=16, d_ff=4096, vocab=40000, dropout=0.3),
}


def param_shapes(enc_layers, dec_layers, d_model, d_ff, vocab, **_):
    """Ordered (name, shape) list.  Linear weights are [out, in]; one vocab x d matrix serves the
    source embedding, the target embedding and the output projection."""
    d, F = d_model, d_ff
    out = [("embed", (vocab, d))]

    def attn(pre, fused):
        if fused:
            out.extend([(pre + "wqkv", (3 * d, d)), (pre + "bqkv", (3 * d,))])
        else:
            out.extend([(pre + "wq", (d, d)), (pre + "bq", (d,)), (pre + "wkv", (2 * d, d)), (pre + "bkv", (2 * d,))])
        out.extend([(pre + "wo", (d, d)), (pre + "bo", (d,))])

    def ln(pre):
        out.extend([(pre + "g", (d,)), (pre + "b", (d,))])

    def ffn(pre):
        out.extend([(pre + "w1", (F, d)), (pre + "b1", (F,)), (pre + "w2", (d, F)), (pre + "b2", (d,))])

    for l in range(enc_layers):
        attn(f"enc{l}.attn.", True); ln(f"enc{l}.ln1."); ffn(f"enc{l}.ffn."); ln(f"enc{l}.ln2.")
    for l in range(dec_layers):
        attn(f"dec{l}.self.", True); ln(f"dec{l}.ln1.")
        attn(f"dec{l}.cross.", False); ln(f"dec{l}.ln2.")
        ffn(f"dec{l}.ffn."); ln(f"dec{l}.ln3.")
    return out


def param_count(**model):
    return sum(int(np.prod(s)) for _, s in param_shapes(**model))


def init_weights(seed=0, perturb=0.0, **model):
    """Xavier-uniform per logical matrix (W_q, W_k, W_v drawn separately), biases 0, LayerNorm
    gain 1 / shift 0, then rounded to fp16 (the value both the fp16 weights and the fp32 master
    start from).  `perturb` > 0 adds uniform noise to biases and LayerNorm parameters so that
    tests exercise them with non-trivial values.  Returns dict name -> float16 array."""
    rng = np.random.default_rng(seed)
    d = model["d_model"]
    W = {}
    for name, shape in param_shapes(**model):
        if len(shape) == 2:
            blocks = []
            rows_left = shape[0]
            # fused projections are stacks of d x d matrices, each with its own fan-out
            blk_rows = d if name.endswith(("wqkv", "wkv")) else shape[0]
            while rows_left > 0:
                bound = np.sqrt(6.0 / (blk_rows + shape[1]))
                blocks.append(rng.uniform(-bound, bound, size=(blk_rows, shape[1])))
                rows_left -= blk_rows
            w = np.concatenate(blocks, axis=0)
        elif name.endswith(".g"):
            w = np.ones(shape) + (rng.uniform(-perturb, perturb, size=shape) if perturb else 0.0)
        else:
            w = rng.uniform(-perturb, perturb, size=shape) if perturb else np.zeros(shape)
        W[name] = w.astype(np.float16)
    return W


# ----------------------------------------------------------------------------------------
# sentences and batches
# ----------------------------------------------------------------------------------------
def _make_batch(src_rows, tgt_rows):
    """Right-pad to the batch maxima; decoder input is the target shifted right behind BOS."""
    B = len(src_rows)
    S = max(len(r) for r in src_rows)
    T = max(len(r) for r in tgt_rows)
    src = np.full((B, S), PAD, dtype=np.int32)
    tgt_in = np.full((B, T), PAD, dtype=np.int32)
    tgt_out = np.full((B, T), PAD, dtype=np.int32)
    for b in range(B):
        s, t = src_rows[b], tgt_rows[b]
        src[b, : len(s)] = s
        tgt_out[b, : len(t)] = t
        tgt_in[b, 0] = BOS
        tgt_in[b, 1: len(t)] = t[:-1]
    return {"src": src, "tgt_in": tgt_in, "tgt_out": tgt_out}


def tiny_batch(seed=1001, B=8, S=16, T=16, vocab=1000, short_rows=2, short_by=5):
    """Configuration 1: B sentence pairs of length S/T, ids uniform in [4, vocab); the last
    `short_rows` rows are `short_by` tokens shorter (right-padded)."""
    rng = np.random.default_rng(seed)
    src_rows, tgt_rows = [], []
    for b in range(B):
        cut = short_by if b >= B - short_rows else 0
        src_rows.append(rng.integers(4, vocab, size=S - cut))
        tgt_rows.append(rng.integers(4, vocab, size=T - cut))
    return _make_batch(src_rows, tgt_rows)


def sample_lengths(rng, n, mean, sigma, lo=1, hi=256):
    """Target lengths ~ lognormal with distribution mean `mean` and log-space sd `sigma`, clipped;
    source length = target length x (1 + U(-0.2, 0.2)), clipped."""
    mu = np.log(mean) - 0.5 * sigma * sigma
    tgt = np.clip(np.rint(rng.lognormal(mu, sigma, size=n)), lo, hi).astype(np.int64)
    src = np.clip(np.rint(tgt * (1.0 + rng.uniform(-0.2, 0.2, size=n))), lo, hi).astype(np.int64)
    return src, tgt


def zipf_sampler(vocab, s=1.1):
    """Finite Zipf over ranks 1..vocab-4 (rank r -> id r+3), sampled by inverse CDF."""
    w = 1.0 / np.power(np.arange(1, vocab - 3, dtype=np.float64), s)
    cdf = np.cumsum(w) / w.sum()

    def draw(rng, n):
        r = np.searchsorted(cdf, rng.random(n), side="left")
        return (np.minimum(r, vocab - 5) + 4).astype(np.int32)

    return draw


def bucket_by_tokens(src_len, tgt_len, max_tokens):
    """Sort sentences by (target length, source length) and cut the sorted list into batches with
    B * max(S, T) <= max_tokens.  Returns a list of index arrays."""
    order = np.lexsort((src_len, tgt_len))
    batches, cur, cur_max = [], [], 0
    for i in order:
        m = max(cur_max, int(src_len[i]), int(tgt_len[i]))
        if cur and (len(cur) + 1) * m > max_tokens:
            batches.append(np.array(cur))
            cur, m = [], max(int(src_len[i]), int(tgt_len[i]))
        cur.append(i)
        cur_max = m
    if cur:
        batches.append(np.array(cur))
    return batches


WORKLOADS = {
    # name: (model, rng seed, max tokens, lognormal mean, sigma)
    "base": ("base", 1002, 3584, 27.0, 0.6),
    "big": ("big", 1003, 3584, 27.0, 0.6),
    "big_accum": ("big", 1004, 3584, 27.0, 0.6),
    "big40k": ("big40k", 1005, 5120, 35.0, 0.7),
}


def make_buckets(workload, n_sentences=200_000):
    """All (B, S, T) buckets of a workload's sentence population, sorted by T.
    Returns (list of index arrays, src_len, tgt_len, rng)."""
    model, seed, max_tok, mean, sigma = WORKLOADS[workload]
    rng = np.random.default_rng(seed)
    src_len, tgt_len = sample_lengths(rng, n_sentences, mean, sigma)
    return bucket_by_tokens(src_len, tgt_len, max_tok), src_len, tgt_len, rng


def fill_batch(idx, src_len, tgt_len, vocab, rng, draw=None):
    draw = draw or zipf_sampler(vocab)
    src_rows = [draw(rng, int(src_len[i])) for i in idx]
    tgt_rows = [draw(rng, int(tgt_len[i])) for i in idx]
    return _make_batch(src_rows, tgt_rows)


def workload_batches(workload, which="median", count=1, n_sentences=200_000):
    """Micro-batches of a workload.  which = "median": `count` consecutive buckets around the
    median bucket; "spread": `count` buckets at evenly spaced percentiles of T; "random":
    `count` buckets drawn uniformly."""
    model = MODELS[WORKLOADS[workload][0]]
    buckets, src_len, tgt_len, rng = make_buckets(workload, n_sentences)
    nb = len(buckets)
    if which == "median":
        first = max(0, nb // 2 - count // 2)
        pick = list(range(first, min(nb, first + count)))
    elif which == "spread":
        pick = [int(round(q * (nb - 1))) for q in np.linspace(0.01, 0.99, count)]
    else:
        pick = list(rng.integers(0, nb, size=count))
    draw = zipf_sampler(model["vocab"])
    return [fill_batch(buckets[i], src_len, tgt_len, model["vocab"], rng, draw) for i in pick]
