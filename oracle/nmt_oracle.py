"""Reference oracle for the reduced-precision Transformer training step.

TEST INFRASTRUCTURE ONLY.  A plain, slow, fp64 numpy implementation of what the
GPU hot path computes: Transformer encoder-decoder forward (model section, "Models and
Hyperparameters"), label-smoothed cross-entropy (same section), loss scaling and
fp16 -> fp32 gradient conversion with overflow detection ("Half-Precision Training"),
gradient accumulation over several sub-batches ("Training with Larger Batches"), and
Adam with the warmup / inverse-sqrt learning-rate schedule (model section).

It shares no code with the HIP library and imports nothing from it.  Only tests,
the smoke check and the benchmark's CPU-baseline leg may import this module.

All arithmetic is float64; logs are natural.  Two precisions of the forward / backward pass:
  * storage="fp64" (default): every tensor stays float64; fp16 *storage* is emulated only where
    it decides the overflow predicate (per-micro-batch gradients rounded to fp16 before they
    are accumulated in wide precision).  This is the form the finite-difference and autograd
    pins check.
  * storage="fp16": the precision "Half-Precision Training" states -- all forward-backward
    computations in FP16, the loss in FP32.  Every tensor one operator hands to the next
    (embedding output, each projection's output, attention probabilities and output, each
    LayerNorm output, logits, and every activation gradient on the way back) is rounded to IEEE
    binary16 (nearest even) where it is produced; sums inside an operator (dot products,
    softmax and LayerNorm statistics, the loss) stay wide.  Binary decisions taken by floating
    point (the ReLU gates) are thereby taken on fp16 values, as the method takes them.

Parity pins (tests/test_oracle_*.py): finite differences of the loss, an independent
torch-autograd model, accumulation equality, padding invariance, loss-scale
invariance, closed forms of the label-smoothed loss, LayerNorm identities, Adam and
schedule closed forms, Philox known-answer vectors; for storage="fp16": the rounding function
against hand-computed binary16 neighbours, every stored tensor exactly representable, identical
results to the fp64 form when nothing needs rounding, and closeness to the fp64 form.
"""
from __future__ import annotations

import math
import numpy as np

# ----------------------------------------------------------------------------------------
# Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3", SC'11)
# ----------------------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: (..., 4) integer array of 32-bit words, key: (2,) 32-bit words.
    Returns (..., 4) uint32 — ten rounds of the Philox-4x32 bijection."""
    c = np.asarray(counter, dtype=np.uint64) & _MASK32
    c0, c1, c2, c3 = (c[..., i].copy() for i in range(4))
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for rnd in range(10):
        if rnd > 0:  # Weyl-sequence key schedule
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0            # 32x32 -> 64 bit products
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


# Dropout sites.  A site id selects an independent random stream.
SITE_EMB_SRC = 0
SITE_EMB_TGT = 1
KIND_SELF_RES, KIND_CROSS_RES, KIND_FFN_ACT, KIND_FFN_RES = 0, 1, 2, 3


def layer_site(layer_index: int, kind: int) -> int:
    """layer_index: encoder layers 0..Le-1, decoder layers Le..Le+Ld-1."""
    return 16 * (1 + layer_index) + kind


def dropout_threshold(p: float) -> int:
    """A 16-bit uniform u is *kept* iff u >= ceil(p * 2^16); p is taken as the float32 value."""
    p32 = float(np.float32(p))
    return int(math.ceil(p32 * 65536.0))


def dropout_keep(seed: int, site: int, step: int, micro: int, sent_uid, n_pos: int,
                 n_cols: int, p: float):
    """Keep-mask (bool [B*n_pos, n_cols]) of the counter-based dropout.

    Element (sentence b, position t, column c) draws from
        Philox4x32-10(counter = (c >> 3, sent_uid[b], site << 16 | t, step << 8 | micro),
                      key = (seed low word, seed high word));
    word (c >> 1) & 3 of the output, 16-bit half (c & 1) (0 = low half), is the uniform.
    The mask therefore depends on the sentence id and the position, never on how a
    batch is padded or split.
    """
    sent_uid = np.asarray(sent_uid, dtype=np.uint64)
    B = sent_uid.shape[0]
    if p <= 0.0:
        return np.ones((B * n_pos, n_cols), dtype=bool)
    n_grp = (n_cols + 7) // 8
    ctr = np.zeros((B, n_pos, n_grp, 4), dtype=np.uint64)
    ctr[..., 0] = np.arange(n_grp, dtype=np.uint64)[None, None, :]
    ctr[..., 1] = sent_uid[:, None, None]
    ctr[..., 2] = (np.uint64(site) << np.uint64(16)) | np.arange(n_pos, dtype=np.uint64)[None, :, None]
    ctr[..., 3] = np.uint64(((int(step) << 8) | int(micro)) & 0xFFFFFFFF)
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = philox4x32_10(ctr, key)                                    # [B, n_pos, n_grp, 4]
    halves = np.stack([words & np.uint32(0xFFFF), words >> np.uint32(16)], axis=-1)  # [...,4,2]
    u16 = halves.reshape(B, n_pos, n_grp * 8)[:, :, :n_cols]
    return (u16 >= np.uint32(dropout_threshold(p))).reshape(B * n_pos, n_cols)


# ----------------------------------------------------------------------------------------
# Building blocks (forward and hand-written reverse mode)
# ----------------------------------------------------------------------------------------
def positional_encoding(n_pos: int, d: int):
    """Sinusoidal positions, interleaved: PE[t, 2i] = sin(t / 10000^(2i/d)), PE[t, 2i+1] = cos(same)."""
    pe = np.zeros((n_pos, d), dtype=np.float64)
    t = np.arange(n_pos, dtype=np.float64)[:, None]
    i2 = np.arange(0, d, 2, dtype=np.float64)[None, :]
    ang = t / np.power(10000.0, i2 / d)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)[:, : d // 2]
    return pe


def linear_fwd(x, W, b=None):
    """y = x W^T (+ b); W is [out, in]."""
    y = x @ W.T
    return y if b is None else y + b


def linear_bwd(x, W, dy):
    return dy @ W, dy.T @ x, dy.sum(axis=0)


def layernorm_fwd(y, gamma, beta, eps):
    """Normalise each row to zero mean / unit (biased) variance, then scale and shift."""
    mu = y.mean(axis=1, keepdims=True)
    var = ((y - mu) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (y - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dout, gamma, saved):
    xhat, rstd = saved
    g = dout * gamma
    dy = rstd * (g - g.mean(axis=1, keepdims=True) - xhat * (g * xhat).mean(axis=1, keepdims=True))
    return dy, (dout * xhat).sum(axis=0), dout.sum(axis=0)


def softmax_rows(a):
    """Row softmax over the last axis; -inf entries get probability exactly 0."""
    m = a.max(axis=-1, keepdims=True)
    e = np.exp(a - m)
    return e / e.sum(axis=-1, keepdims=True)


def _split_heads(x, B, T, h):
    return x.reshape(B, T, h, -1).transpose(0, 2, 1, 3)          # [B,h,T,dh]


def _merge_heads(x):
    B, h, T, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * T, h * dh)


def attention_fwd(q, k, v, masked, B, Tq, Tk, h, stored=None):
    """q [B*Tq,d], k,v [B*Tk,d]; masked: bool [B,Tq,Tk], True = this key may not be seen.
    stored: rounding applied to the probabilities where they are handed to the product with V
    (None: none)."""
    dh = q.shape[1] // h
    qh, kh, vh = _split_heads(q, B, Tq, h), _split_heads(k, B, Tk, h), _split_heads(v, B, Tk, h)
    a = qh @ kh.transpose(0, 1, 3, 2) / math.sqrt(dh)
    a = np.where(masked[:, None, :, :], -np.inf, a)
    p = softmax_rows(a)
    if stored is not None:
        p = stored(p)
    o = p @ vh
    return _merge_heads(o), (qh, kh, vh, p)


def attention_bwd(do, saved, B, Tq, Tk, h):
    qh, kh, vh, p = saved
    dh = qh.shape[-1]
    doh = _split_heads(do, B, Tq, h)
    dv = p.transpose(0, 1, 3, 2) @ doh
    dp = doh @ vh.transpose(0, 1, 3, 2)
    da = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    da = da / math.sqrt(dh)
    dq = da @ kh
    dk = da.transpose(0, 1, 3, 2) @ qh
    return _merge_heads(dq), _merge_heads(dk), _merge_heads(dv)


def label_smoothed_nll(z, y, pad_id, eps):
    """Per-row loss against q = (1-eps) onehot(y) + eps/V (uniform prior over all V symbols),
    summed over rows whose target is not padding.  Returns (loss_sum, n_tok, dz) where
    dz = softmax(z) - q on counted rows and 0 elsewhere."""
    N, V = z.shape
    m = z.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(z - m).sum(axis=1))
    live = (y != pad_id)
    zy = z[np.arange(N), y]
    row = lse - (1.0 - eps) * zy - (eps / V) * z.sum(axis=1)
    loss_sum = float(row[live].sum())
    p = np.exp(z - lse[:, None])
    q = np.full((N, V), eps / V)
    q[np.arange(N), y] += 1.0 - eps
    dz = (p - q) * live[:, None]
    return loss_sum, int(live.sum()), dz


# ----------------------------------------------------------------------------------------
# The model
# ----------------------------------------------------------------------------------------
class Config:
    """Plain holder of the model hyper-parameters (names follow the model section)."""

    def __init__(self, enc_layers, dec_layers, d_model, n_heads, d_ff, vocab, pad_id=1,
                 dropout=0.0, act_dropout=0.0, label_smoothing=0.1, ln_eps=1e-5, seed=0):
        self.enc_layers, self.dec_layers = enc_layers, dec_layers
        self.d_model, self.n_heads, self.d_ff, self.vocab = d_model, n_heads, d_ff, vocab
        self.pad_id = pad_id
        self.dropout, self.act_dropout = dropout, act_dropout
        self.label_smoothing, self.ln_eps, self.seed = label_smoothing, ln_eps, seed


def _drop(x, keep, p):
    if p <= 0.0:
        return x
    return x * keep / (1.0 - float(np.float32(p)))


def fp16_round(x):
    """IEEE binary16 round-to-nearest-even of every element (|x| >= 65520 -> +-inf), widened again."""
    with np.errstate(over="ignore"):
        return np.asarray(x).astype(np.float16).astype(np.float64)


def _identity(x):
    return x


def _stored(storage: str):
    """What happens to a tensor where one operator hands it to the next."""
    if storage == "fp64":
        return _identity
    if storage == "fp16":
        return fp16_round
    raise ValueError(f"storage must be 'fp64' or 'fp16', not {storage!r}")


def _sublayer_out(resid, sub, keep, p, gamma, beta, eps):
    """x <- LayerNorm(x + Dropout(Sublayer(x))): normalisation after the residual."""
    return layernorm_fwd(resid + _drop(sub, keep, p), gamma, beta, eps)


def forward_loss(P, cfg: Config, src, tgt_in, tgt_out, *, training=True, step=0, micro=0,
                 sent_uid=None, storage="fp64"):
    """One forward pass and the (unscaled) label-smoothed loss.

    P: dict name -> float64 array (values of the fp16 weights).  src [B,S], tgt_in / tgt_out
    [B,T]: int ids, right-padded with cfg.pad_id.  storage: "fp64", or "fp16" to round every
    tensor handed from one operator to the next to binary16 ("Half-Precision Training"; see the
    module header).  Returns (loss_sum in nats, n_tok, cache); backward() follows the cache's mode.
    """
    st = _stored(storage)
    src, tgt_in, tgt_out = (np.asarray(a, dtype=np.int64) for a in (src, tgt_in, tgt_out))
    B, S = src.shape
    T = tgt_in.shape[1]
    d, h, Le, Ld = cfg.d_model, cfg.n_heads, cfg.enc_layers, cfg.dec_layers
    p_res = cfg.dropout if training else 0.0
    p_act = cfg.act_dropout if training else 0.0
    uid = np.arange(B) if sent_uid is None else np.asarray(sent_uid)

    def keep(site, n_pos, n_cols, p):
        return dropout_keep(cfg.seed, site, step, micro, uid, n_pos, n_cols, p)

    E = P["embed"]
    cache = {"B": B, "S": S, "T": T, "src": src, "tgt_in": tgt_in, "tgt_out": tgt_out,
             "p_res": p_res, "p_act": p_act, "enc": [], "dec": [], "storage": storage}
    att_st = None if storage == "fp64" else st

    src_pad = (src == cfg.pad_id)                                    # [B,S]
    tgt_pad = (tgt_in == cfg.pad_id)                                 # [B,T]
    enc_mask = np.broadcast_to(src_pad[:, None, :], (B, S, S))
    cross_mask = np.broadcast_to(src_pad[:, None, :], (B, T, S))
    future = np.triu(np.ones((T, T), dtype=bool), k=1)               # key j > query i
    self_mask = future[None, :, :] | tgt_pad[:, None, :]

    # ---- encoder -----------------------------------------------------------------
    k_es = keep(SITE_EMB_SRC, S, d, p_res)
    x = st(_drop(math.sqrt(d) * E[src.reshape(-1)] + np.tile(positional_encoding(S, d), (B, 1)), k_es, p_res))
    cache["keep_emb_src"] = k_es
    for l in range(Le):
        pre = f"enc{l}."
        c = {"x_in": x}
        qkv = st(linear_fwd(x, P[pre + "attn.wqkv"], P[pre + "attn.bqkv"]))
        o, c["attn"] = attention_fwd(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], enc_mask, B, S, S, h, att_st)
        o = st(o)
        c["o"] = o
        s1 = st(linear_fwd(o, P[pre + "attn.wo"], P[pre + "attn.bo"]))
        c["keep1"] = keep(layer_site(l, KIND_SELF_RES), S, d, p_res)
        x1, c["ln1"] = _sublayer_out(x, s1, c["keep1"], p_res, P[pre + "ln1.g"], P[pre + "ln1.b"], cfg.ln_eps)
        x1 = st(x1)
        c["x1"] = x1
        hpre = linear_fwd(x1, P[pre + "ffn.w1"], P[pre + "ffn.b1"])
        c["keep_act"] = keep(layer_site(l, KIND_FFN_ACT), S, cfg.d_ff, p_act)
        c["relu"] = st(np.maximum(hpre, 0.0))      # what the gate of the backward pass looks at
        hact = st(_drop(np.maximum(hpre, 0.0), c["keep_act"], p_act))
        c["hpre"], c["hact"] = hpre, hact
        s2 = st(linear_fwd(hact, P[pre + "ffn.w2"], P[pre + "ffn.b2"]))
        c["keep2"] = keep(layer_site(l, KIND_FFN_RES), S, d, p_res)
        x, c["ln2"] = _sublayer_out(x1, s2, c["keep2"], p_res, P[pre + "ln2.g"], P[pre + "ln2.b"], cfg.ln_eps)
        x = st(x)
        cache["enc"].append(c)
    enc_out = x
    cache["enc_out"] = enc_out

    # ---- decoder -----------------------------------------------------------------
    k_et = keep(SITE_EMB_TGT, T, d, p_res)
    x = st(_drop(math.sqrt(d) * E[tgt_in.reshape(-1)] + np.tile(positional_encoding(T, d), (B, 1)), k_et, p_res))
    cache["keep_emb_tgt"] = k_et
    for l in range(Ld):
        pre = f"dec{l}."
        li = Le + l
        c = {"x_in": x}
        qkv = st(linear_fwd(x, P[pre + "self.wqkv"], P[pre + "self.bqkv"]))
        o, c["self"] = attention_fwd(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], self_mask, B, T, T, h, att_st)
        o = st(o)
        c["o_self"] = o
        s1 = st(linear_fwd(o, P[pre + "self.wo"], P[pre + "self.bo"]))
        c["keep1"] = keep(layer_site(li, KIND_SELF_RES), T, d, p_res)
        x1, c["ln1"] = _sublayer_out(x, s1, c["keep1"], p_res, P[pre + "ln1.g"], P[pre + "ln1.b"], cfg.ln_eps)
        x1 = st(x1)
        c["x1"] = x1
        q = st(linear_fwd(x1, P[pre + "cross.wq"], P[pre + "cross.bq"]))
        kv = st(linear_fwd(enc_out, P[pre + "cross.wkv"], P[pre + "cross.bkv"]))
        o, c["cross"] = attention_fwd(q, kv[:, :d], kv[:, d:], cross_mask, B, T, S, h, att_st)
        o = st(o)
        c["o_cross"] = o
        s2 = st(linear_fwd(o, P[pre + "cross.wo"], P[pre + "cross.bo"]))
        c["keep2"] = keep(layer_site(li, KIND_CROSS_RES), T, d, p_res)
        x2, c["ln2"] = _sublayer_out(x1, s2, c["keep2"], p_res, P[pre + "ln2.g"], P[pre + "ln2.b"], cfg.ln_eps)
        x2 = st(x2)
        c["x2"] = x2
        hpre = linear_fwd(x2, P[pre + "ffn.w1"], P[pre + "ffn.b1"])
        c["keep_act"] = keep(layer_site(li, KIND_FFN_ACT), T, cfg.d_ff, p_act)
        c["relu"] = st(np.maximum(hpre, 0.0))
        hact = st(_drop(np.maximum(hpre, 0.0), c["keep_act"], p_act))
        c["hpre"], c["hact"] = hpre, hact
        s3 = st(linear_fwd(hact, P[pre + "ffn.w2"], P[pre + "ffn.b2"]))
        c["keep3"] = keep(layer_site(li, KIND_FFN_RES), T, d, p_res)
        x, c["ln3"] = _sublayer_out(x2, s3, c["keep3"], p_res, P[pre + "ln3.g"], P[pre + "ln3.b"], cfg.ln_eps)
        x = st(x)
        cache["dec"].append(c)
    cache["dec_out"] = x

    # ---- output projection (tied to the embedding) and loss ------------------------
    z = st(x @ E.T)
    loss_sum, n_tok, dz = label_smoothed_nll(z, tgt_out.reshape(-1), cfg.pad_id, cfg.label_smoothing)
    cache["logits"] = z
    cache["dz_unit"] = dz
    return loss_sum, n_tok, cache


def backward(P, cfg: Config, cache, loss_scale: float, gates=None):
    """Gradient of loss_scale * loss_sum with respect to every parameter (dict of float64), in the
    storage mode of the forward pass that made `cache`: with "fp16" every activation gradient is
    rounded to binary16 where one operator hands it to the next (a residual fan-in is one operator:
    the two branches are added wide and the sum is rounded), the weight gradients are formed wide
    from those rounded tensors (their own rounding is to_fp16_storage's business).

    gates (tests only): dict "enc0.ffn." / "dec1.ffn." ... -> bool array [N, d_ff] of ReLU decisions to
    differentiate through instead of this pass's own (pre-activation > 0).  A gate whose pre-activation is
    smaller than the rounding effects of reduced-precision arithmetic has no unique decision; a test that
    compares gradients of two implementations first checks that they differ on such gates only
    (undecided_relu_gates) and then compares the gradients for one and the same set of decisions."""
    B, S, T = cache["B"], cache["S"], cache["T"]
    d, h, Le, Ld = cfg.d_model, cfg.n_heads, cfg.enc_layers, cfg.dec_layers
    p_res, p_act = cache["p_res"], cache["p_act"]
    st = _stored(cache.get("storage", "fp64"))
    G = {name: np.zeros_like(val) for name, val in P.items()}
    E = P["embed"]

    dz = st(cache["dz_unit"] * loss_scale)
    G["embed"] += dz.T @ cache["dec_out"]
    dx = st(dz @ E)
    d_enc_out = None

    def ffn_bwd(pre, c, x_in, dsub):
        """dsub: gradient at the FFN output (after residual dropout was undone). Returns d x_in
        (wide: the caller adds the residual branch before the sum is stored)."""
        dh, G[pre + "ffn.w2"], G[pre + "ffn.b2"] = linear_bwd(c["hact"], P[pre + "ffn.w2"], dsub)
        gate = c["relu"] > 0.0
        if gates is not None and pre + "ffn." in gates:
            gate = np.asarray(gates[pre + "ffn."], dtype=bool).reshape(gate.shape)
        dh = st(_drop(dh, c["keep_act"], p_act) * gate)
        dxi, G[pre + "ffn.w1"], G[pre + "ffn.b1"] = linear_bwd(x_in, P[pre + "ffn.w1"], dh)
        return dxi

    def attn_bwd(c_attn, do, Tq, Tk):
        dq, dk, dv = attention_bwd(do, c_attn, B, Tq, Tk, h)
        return st(dq), st(dk), st(dv)

    for l in reversed(range(Ld)):
        pre = f"dec{l}."
        c = cache["dec"][l]
        dy, G[pre + "ln3.g"], G[pre + "ln3.b"] = layernorm_bwd(dx, P[pre + "ln3.g"], c["ln3"])
        dy = st(dy)
        dx2 = st(dy + ffn_bwd(pre, c, c["x2"], st(_drop(dy, c["keep3"], p_res))))
        # encoder-decoder attention
        dy, G[pre + "ln2.g"], G[pre + "ln2.b"] = layernorm_bwd(dx2, P[pre + "ln2.g"], c["ln2"])
        dy = st(dy)
        do, G[pre + "cross.wo"], G[pre + "cross.bo"] = linear_bwd(c["o_cross"], P[pre + "cross.wo"],
                                                                  st(_drop(dy, c["keep2"], p_res)))
        dq, dk, dv = attn_bwd(c["cross"], st(do), T, S)
        dx1q, G[pre + "cross.wq"], G[pre + "cross.bq"] = linear_bwd(c["x1"], P[pre + "cross.wq"], dq)
        dkv = np.concatenate([dk, dv], axis=1)
        de, G[pre + "cross.wkv"], G[pre + "cross.bkv"] = linear_bwd(cache["enc_out"], P[pre + "cross.wkv"], dkv)
        d_enc_out = st(de) if d_enc_out is None else st(d_enc_out + de)   # every decoder layer reads the encoder output
        dx1 = st(dy + dx1q)
        # masked self-attention
        dy, G[pre + "ln1.g"], G[pre + "ln1.b"] = layernorm_bwd(dx1, P[pre + "ln1.g"], c["ln1"])
        dy = st(dy)
        do, G[pre + "self.wo"], G[pre + "self.bo"] = linear_bwd(c["o_self"], P[pre + "self.wo"],
                                                                st(_drop(dy, c["keep1"], p_res)))
        dq, dk, dv = attn_bwd(c["self"], st(do), T, T)
        dqkv = np.concatenate([dq, dk, dv], axis=1)
        dxi, G[pre + "self.wqkv"], G[pre + "self.bqkv"] = linear_bwd(c["x_in"], P[pre + "self.wqkv"], dqkv)
        dx = st(dy + dxi)
    # target embedding: x = drop(sqrt(d) E[id] + PE)
    demb = _drop(dx, cache["keep_emb_tgt"], p_res) * math.sqrt(d)
    np.add.at(G["embed"], cache["tgt_in"].reshape(-1), demb)

    dx = d_enc_out
    for l in reversed(range(Le)):
        pre = f"enc{l}."
        c = cache["enc"][l]
        dy, G[pre + "ln2.g"], G[pre + "ln2.b"] = layernorm_bwd(dx, P[pre + "ln2.g"], c["ln2"])
        dy = st(dy)
        dx1 = st(dy + ffn_bwd(pre, c, c["x1"], st(_drop(dy, c["keep2"], p_res))))
        dy, G[pre + "ln1.g"], G[pre + "ln1.b"] = layernorm_bwd(dx1, P[pre + "ln1.g"], c["ln1"])
        dy = st(dy)
        do, G[pre + "attn.wo"], G[pre + "attn.bo"] = linear_bwd(c["o"], P[pre + "attn.wo"],
                                                                st(_drop(dy, c["keep1"], p_res)))
        dq, dk, dv = attn_bwd(c["attn"], st(do), S, S)
        dqkv = np.concatenate([dq, dk, dv], axis=1)
        dxi, G[pre + "attn.wqkv"], G[pre + "attn.bqkv"] = linear_bwd(c["x_in"], P[pre + "attn.wqkv"], dqkv)
        dx = st(dy + dxi)
    demb = _drop(dx, cache["keep_emb_src"], p_res) * math.sqrt(d)
    np.add.at(G["embed"], cache["src"].reshape(-1), demb)
    return G


def undecided_relu_gates(P, cfg: Config, cache, width=8.0):
    """Per feed-forward layer ("enc0.ffn." ...): bool [N, d_ff], True where the sign of the pre-activation
    is not decided at fp16 precision: |x W1^T + b1| <= width * 2^-11 * sqrt(sum_k (x_k W1_jk)^2), i.e. within
    `width` times the rms effect of rounding each term of the dot product to 11 significant bits (binary16
    keeps 11; the layer input has been through that rounding at every operator before it)."""
    out = {}
    for side, key_x in (("enc", "x1"), ("dec", "x2")):
        for l, c in enumerate(cache[side]):
            pre = f"{side}{l}.ffn."
            x, W1 = c[key_x], P[pre + "w1"]
            out[pre] = np.abs(c["hpre"]) <= width * 2.0 ** -11 * np.sqrt((x * x) @ (W1 * W1).T)
    return out


# ----------------------------------------------------------------------------------------
# Reduced-precision bookkeeping, accumulation, update
# ----------------------------------------------------------------------------------------
def to_fp16_storage(G):
    """Round each gradient to IEEE binary16 (nearest even; |x| >= 65520 becomes +-inf) and
    widen again: the value a 16-bit gradient buffer would hold."""
    return {k: fp16_round(v) for k, v in G.items()}


def accumulate(acc, g16, first: bool):
    """acc <- g16 (first micro-batch of an update) or acc <- acc + g16."""
    with np.errstate(invalid="ignore"):
        if first or acc is None:
            return {k: v.copy() for k, v in g16.items()}
        return {k: acc[k] + g16[k] for k in g16}


def check_overflow(acc, inv_scale: float):
    """Overflow iff any accumulated element is inf or NaN.  Returns (flag, unscaled grads)."""
    flag = int(any(not np.isfinite(v).all() for v in acc.values()))
    with np.errstate(invalid="ignore", over="ignore"):
        return flag, {k: v * inv_scale for k, v in acc.items()}


def adam_step(master, m, v, g, lr, beta1, beta2, eps, t, flag):
    """Adam (Kingma & Ba, Algorithm 1) on the wide-precision master weights, in place;
    t is 1-based.  A set overflow flag turns the call into a no-op.  Returns the fp16 copy of
    the weights (as float64 values)."""
    if not flag:
        for k in master:
            m[k] = beta1 * m[k] + (1.0 - beta1) * g[k]
            v[k] = beta2 * v[k] + (1.0 - beta2) * g[k] * g[k]
            mhat = m[k] / (1.0 - beta1 ** t)
            vhat = v[k] / (1.0 - beta2 ** t)
            master[k] = master[k] - lr * mhat / (np.sqrt(vhat) + eps)
    return {k: w.astype(np.float16).astype(np.float64) for k, w in master.items()}


def lr_schedule(t: int, peak: float, warmup: int = 4000):
    """Linear warm-up from 0 to `peak` over `warmup` updates, then proportional to 1/sqrt(t)."""
    return peak * min(t / warmup, math.sqrt(warmup / t))


class LossScaler:
    """Dynamic loss scaling: halve on overflow, double after `window` overflow-free updates."""

    def __init__(self, init_scale=128.0, window=2000, min_scale=2.0 ** -14):
        self.scale, self.window, self.min_scale, self.clean = float(init_scale), window, min_scale, 0

    def update(self, overflow: bool):
        if overflow:
            self.scale = self.scale / 2.0
            self.clean = 0
            if self.scale < self.min_scale:
                raise FloatingPointError("loss scale fell below its floor")
        else:
            self.clean += 1
            if self.clean == self.window:
                self.scale *= 2.0
                self.clean = 0


def train_update(P16, master, m, v, cfg, micro_batches, scaler: LossScaler, t, lr, betas=(0.9, 0.98),
                 eps=1e-8, step=None, scale_override=None, storage="fp64"):
    """One weight update from k micro-batches.  Returns dict with loss, n_tok, flag and the new
    fp16 weights.  `t` is the 1-based Adam step to use if the update is applied."""
    step = t if step is None else step
    S_loss = scaler.scale if scale_override is None else scale_override
    acc, loss_tot, ntok_tot = None, 0.0, 0
    for j, mb in enumerate(micro_batches):
        loss, ntok, cache = forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], training=True,
                                         step=step, micro=j, sent_uid=mb.get("sent_uid"), storage=storage)
        g16 = to_fp16_storage(backward(P16, cfg, cache, S_loss))
        acc = accumulate(acc, g16, j == 0)
        loss_tot += loss
        ntok_tot += ntok
    flag, g = check_overflow(acc, 1.0 / (S_loss * ntok_tot))
    new16 = adam_step(master, m, v, g, lr, betas[0], betas[1], eps, t, flag)
    scaler.update(bool(flag))
    return {"loss_sum": loss_tot, "n_tok": ntok_tot, "flag": flag, "w16": new16, "grad": g, "acc": acc}
