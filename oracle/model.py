"""CPU oracle of the checkpointed training step (TEST INFRASTRUCTURE ONLY).

This file is test infrastructure: only tests, the smoke check and the bench's
cpu_baseline leg may import it.  It shares no code with the HIP library.

What it computes.  Layer-granular activation checkpointing (paper Section 1 and
Section 5: a dropped layer keeps only its boundary tensor and its forward is
replayed in backward) does not change the numerical result of a training
iteration (Section 6.6), so the oracle of the numeric path is the plain
definition: the mean token cross-entropy of a transformer stack and its exact
gradient with respect to every parameter, written with numpy array operations
in the obvious order (materialised L x L attention, no blocking, no fusion).
The iteration structure - forward keeping activations, loss, backward consuming
them - follows Section 2.1.  The model equations are the public BERT / GPT-2
block definitions that the paper's evaluation (Section 6.1) refers to:

  post-LN block:  u  = LN1(h + Attn(h) Wo^T + bo)
                  h' = LN2(u + GELU(u W1^T + b1) W2^T + b2)
  pre-LN block:   u  = h + Attn(LN1(h)) Wo^T + bo
                  h' = u + GELU(LN2(u) W1^T + b1) W2^T + b2      (+ final LN)

Default precision is float64; float32 can be requested.

Pins (tests/test_oracle_model.py): central finite differences on every
parameter tensor, an independent re-derivation through torch CPU autograd over
torch's own library ops, closed-form loss at initialisation, softmax / LN / CE
invariants, L = 1 attention, causal independence, and bitwise equality of
gradients across all checkpoint plans.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf

from . import philox


@dataclass
class Cfg:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_seq: int
    causal: int = 0
    pre_ln: int = 0
    gelu_tanh: int = 0
    head: int = 1
    ln_eps: float = 1e-5
    ffn_by_layer: tuple = ()      # feed-forward width of each layer when they differ (empty: ffn)

    @staticmethod
    def from_shape(d: dict) -> "Cfg":
        keys = ("n_layers", "hidden", "n_heads", "ffn", "vocab", "max_seq",
                "causal", "pre_ln", "gelu_tanh", "head", "ln_eps")
        return Cfg(**{k: d[k] for k in keys}, ffn_by_layer=tuple(d.get("ffn_by_layer", ()) or ()))


@dataclass
class Dropout:
    """Dropout as the fine-tuning tasks of Section 6.1 use it: p_hidden on the embedding output, on
    the attention block's output projection and on the feed-forward block's output (each before
    its residual sum), p_attn on the attention probabilities.  Masks come from a counter-based
    generator keyed by (seed, step), see oracle/philox.py."""
    p_hidden: float = 0.0
    p_attn: float = 0.0
    seed: int = 0
    step: int = 0


# --------------------------------------------------------------------------
# bf16 rounding of inputs (round to nearest, ties to even), so that the oracle
# consumes the same parameter values a bf16 device path stores.
# --------------------------------------------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(f.shape)


# --------------------------------------------------------------------------
# Elementary operations, each with its hand-derived reverse.
# --------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased variance
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, saved, gamma):
    xhat, rstd = saved
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    dxhat = dy * gamma
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma, dbeta


def gelu_fwd(x, tanh_form):
    if tanh_form:
        c = np.sqrt(2.0 / np.pi)
        return 0.5 * x * (1.0 + np.tanh(c * (x + 0.044715 * x ** 3)))
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_grad(x, tanh_form):
    if tanh_form:
        c = np.sqrt(2.0 / np.pi)
        inner = c * (x + 0.044715 * x ** 3)
        t = np.tanh(inner)
        return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * c * (1.0 + 3 * 0.044715 * x * x)
    cdf = 0.5 * (1.0 + _erf(x / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return cdf + x * pdf


def linear_fwd(x, W, b):
    """y = x W^T + b with W stored [out, in]."""
    y = x @ W.T
    if b is not None:
        y = y + b
    return y


def linear_bwd(dy, x, W):
    return dy @ W, dy.T @ x, dy.sum(axis=0)          # dx, dW, db


def split_heads(x, B, L, h):
    d = x.shape[-1] // h
    return x.reshape(B, L, h, d).transpose(0, 2, 1, 3)      # [B,h,L,d]


def merge_heads(x):
    B, h, L, d = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * L, h * d)


def attention_fwd(q, k, v, causal, lengths=None, keep=None):
    """q, k, v: [B,h,L,d].  Returns o and the probability matrix.

    keep (optional, [B,h,L,L]): dropout multipliers of the probabilities (0 or 1/(1-p)); the
    output is (p * keep) v, the returned probabilities are the undropped ones.

    lengths (optional, [B]): sample b has lengths[b] real tokens, the rest of its row is padding
    (the batch is padded to its longest sample, Section 2.1); padded keys get no weight."""
    d = q.shape[-1]
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(float(d))
    L = q.shape[2]
    if causal:
        mask = np.triu(np.ones((L, L), dtype=bool), k=1)
        s = np.where(mask, -np.inf, s)
    if lengths is not None:
        pad = np.arange(L)[None, :] >= np.asarray(lengths)[:, None]          # [B, L] keys that are padding
        s = np.where(pad[:, None, None, :], -np.inf, s)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=-1, keepdims=True)
    return (p if keep is None else p * keep) @ v, p


def attention_bwd(do, q, k, v, p, keep=None):
    d = q.shape[-1]
    pd = p if keep is None else p * keep
    dv = pd.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    if keep is not None:
        dp = dp * keep
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    ds = ds / np.sqrt(float(d))
    dq = ds @ k
    dk = ds.transpose(0, 1, 3, 2) @ q
    return dq, dk, dv


def cross_entropy(logits, labels):
    """Mean over positions with label >= 0 of -log softmax(logits)[label]."""
    valid = labels >= 0
    n = int(valid.sum())
    m = logits.max(axis=-1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(logits - m).sum(axis=-1))
    rows = np.nonzero(valid)[0]
    picked = logits[rows, labels[rows]]
    loss = float((lse[rows] - picked).sum() / max(n, 1))
    dlogits = np.exp(logits - lse[:, None])
    dlogits[rows, labels[rows]] -= 1.0
    dlogits[~valid] = 0.0
    dlogits = dlogits / max(n, 1)
    return loss, dlogits


# --------------------------------------------------------------------------
# One transformer block.
# --------------------------------------------------------------------------
def layer_forward(cfg: Cfg, P: Dict[str, np.ndarray], l: int, h, B: int, L: int, lengths=None, dropout=None):
    pre = f"layer{l}."
    H, nh = cfg.hidden, cfg.n_heads
    S = {"h": h}
    # dropout multipliers of this layer's three sites; a rebuilt layer gets the same ones because
    # they depend on (seed, step, site, element number) only
    S["keep_p"] = S["keep_o"] = S["keep_f"] = None
    if dropout is not None and dropout.p_attn > 0:
        S["keep_p"] = philox.keep_scale(philox.attn_index(B, nh, L), dropout.p_attn, dropout.seed,
                                        philox.site_attn_prob(l), dropout.step, h.dtype.type)
    if dropout is not None and dropout.p_hidden > 0:
        idx = philox.hidden_index(B * L, H)
        S["keep_o"] = philox.keep_scale(idx, dropout.p_hidden, dropout.seed, philox.site_attn_out(l),
                                        dropout.step, h.dtype.type)
        S["keep_f"] = philox.keep_scale(idx, dropout.p_hidden, dropout.seed, philox.site_ffn_out(l),
                                        dropout.step, h.dtype.type)
    a = h
    if cfg.pre_ln:
        a, S["ln1"] = layernorm_fwd(h, P[pre + "ln1_g"], P[pre + "ln1_b"], cfg.ln_eps)
    S["a"] = a
    qkv = linear_fwd(a, P[pre + "wqkv"], P[pre + "bqkv"])
    q = split_heads(qkv[:, :H], B, L, nh)
    k = split_heads(qkv[:, H:2 * H], B, L, nh)
    v = split_heads(qkv[:, 2 * H:], B, L, nh)
    o, p = attention_fwd(q, k, v, cfg.causal, lengths, S["keep_p"])
    S.update(q=q, k=k, v=v, p=p)
    ctx = merge_heads(o)
    S["ctx"] = ctx
    proj = linear_fwd(ctx, P[pre + "wo"], P[pre + "bo"])
    s1 = h + (proj if S["keep_o"] is None else proj * S["keep_o"])
    if cfg.pre_ln:
        u = s1
        f_in, S["ln2"] = layernorm_fwd(u, P[pre + "ln2_g"], P[pre + "ln2_b"], cfg.ln_eps)
    else:
        u, S["ln1"] = layernorm_fwd(s1, P[pre + "ln1_g"], P[pre + "ln1_b"], cfg.ln_eps)
        f_in = u
    S["f_in"] = f_in
    pa = linear_fwd(f_in, P[pre + "w1"], P[pre + "b1"])
    g = gelu_fwd(pa, cfg.gelu_tanh)
    S.update(pa=pa, g=g)
    ffn = linear_fwd(g, P[pre + "w2"], P[pre + "b2"])
    s2 = u + (ffn if S["keep_f"] is None else ffn * S["keep_f"])
    if cfg.pre_ln:
        out = s2
    else:
        out, S["ln2"] = layernorm_fwd(s2, P[pre + "ln2_g"], P[pre + "ln2_b"], cfg.ln_eps)
    return out, S


def layer_backward(cfg: Cfg, P, l: int, S, dout, G: Dict[str, np.ndarray]):
    pre = f"layer{l}."
    H = cfg.hidden
    if cfg.pre_ln:
        ds2 = dout
    else:
        ds2, G[pre + "ln2_g"], G[pre + "ln2_b"] = layernorm_bwd(dout, S["ln2"], P[pre + "ln2_g"])
    dffn = ds2 if S["keep_f"] is None else ds2 * S["keep_f"]
    dg, G[pre + "w2"], G[pre + "b2"] = linear_bwd(dffn, S["g"], P[pre + "w2"])
    dpa = dg * gelu_grad(S["pa"], cfg.gelu_tanh)
    dfin, G[pre + "w1"], G[pre + "b1"] = linear_bwd(dpa, S["f_in"], P[pre + "w1"])
    if cfg.pre_ln:
        dln, G[pre + "ln2_g"], G[pre + "ln2_b"] = layernorm_bwd(dfin, S["ln2"], P[pre + "ln2_g"])
        ds1 = ds2 + dln
    else:
        du = ds2 + dfin
        ds1, G[pre + "ln1_g"], G[pre + "ln1_b"] = layernorm_bwd(du, S["ln1"], P[pre + "ln1_g"])
    dproj = ds1 if S["keep_o"] is None else ds1 * S["keep_o"]
    dctx, G[pre + "wo"], G[pre + "bo"] = linear_bwd(dproj, S["ctx"], P[pre + "wo"])
    B, nh, L, d = S["q"].shape
    do = split_heads(dctx, B, L, nh)
    dq, dk, dv = attention_bwd(do, S["q"], S["k"], S["v"], S["p"], S["keep_p"])
    dqkv = np.concatenate([merge_heads(dq), merge_heads(dk), merge_heads(dv)], axis=1)
    da, G[pre + "wqkv"], G[pre + "bqkv"] = linear_bwd(dqkv, S["a"], P[pre + "wqkv"])
    if cfg.pre_ln:
        dln, G[pre + "ln1_g"], G[pre + "ln1_b"] = layernorm_bwd(da, S["ln1"], P[pre + "ln1_g"])
        return ds1 + dln
    return ds1 + da


# --------------------------------------------------------------------------
# The whole training step.
# --------------------------------------------------------------------------
def train_step(cfg: Cfg, params: Dict[str, np.ndarray], tokens: np.ndarray,
               labels: np.ndarray, plan: int = 0, dtype=np.float64,
               return_logits: bool = False, lengths=None, dropout: "Dropout" = None):
    """Loss and gradients for one mini-batch.

    plan: bitmask, bit l set = layer l drops its activations after its forward
    (only its input survives) and rebuilds them at the start of its backward.
    lengths (optional, [B]): real tokens per sample of a batch padded to L; padded keys are
    masked in every attention and padded positions carry no label.
    dropout (optional): see Dropout; None or zero probabilities leave every value as it is.
    """
    P = {k: np.asanyarray(v, dtype=dtype) for k, v in params.items()}
    B, L = tokens.shape
    T = B * L
    H = cfg.hidden
    ids = tokens.reshape(T)
    lab = labels.reshape(T)
    if lengths is not None:
        lengths = np.asarray(lengths)
        lab = np.where((np.arange(L)[None, :] >= lengths[:, None]).reshape(T), -1, lab)
    pos = np.tile(np.arange(L), B)

    # embedding stage
    emb = P["tok_emb"][ids] + P["pos_emb"][pos]
    if cfg.pre_ln:
        h = emb
        emb_saved = None
    else:
        h, emb_saved = layernorm_fwd(emb, P["emb_ln_g"], P["emb_ln_b"], cfg.ln_eps)
    keep_e = None
    if dropout is not None and dropout.p_hidden > 0:
        keep_e = philox.keep_scale(philox.hidden_index(T, H), dropout.p_hidden, dropout.seed,
                                   philox.SITE_EMBED, dropout.step, h.dtype.type)
        h = h * keep_e

    # layer stack, keeping or dropping activations
    inputs: List[np.ndarray] = []
    saved: List[Optional[dict]] = []
    for l in range(cfg.n_layers):
        inputs.append(h)
        h, S = layer_forward(cfg, P, l, h, B, L, lengths, dropout)
        saved.append(None if (plan >> l) & 1 else S)

    # head and loss
    hs = h
    if cfg.pre_ln:
        hs, fin_saved = layernorm_fwd(h, P["final_ln_g"], P["final_ln_b"], cfg.ln_eps)
    if cfg.head:
        z = linear_fwd(hs, P["head.wt"], P["head.bt"])
        gz = gelu_fwd(z, cfg.gelu_tanh)
        t, head_ln = layernorm_fwd(gz, P["head.ln_g"], P["head.ln_b"], cfg.ln_eps)
        logits = t @ P["tok_emb"].T + P["head.bdec"]
    else:
        t = hs
        logits = t @ P["tok_emb"].T
    loss, dlogits = cross_entropy(logits, lab)

    G: Dict[str, np.ndarray] = {}
    # head backward (the tied decoder's contribution to tok_emb comes first)
    G["tok_emb"] = dlogits.T @ t
    dt = dlogits @ P["tok_emb"]
    if cfg.head:
        G["head.bdec"] = dlogits.sum(axis=0)
        dgz, G["head.ln_g"], G["head.ln_b"] = layernorm_bwd(dt, head_ln, P["head.ln_g"])
        dz = dgz * gelu_grad(z, cfg.gelu_tanh)
        dh, G["head.wt"], G["head.bt"] = linear_bwd(dz, hs, P["head.wt"])
    else:
        dh = dt
    if cfg.pre_ln:
        dh, G["final_ln_g"], G["final_ln_b"] = layernorm_bwd(dh, fin_saved, P["final_ln_g"])

    # layer stack in reverse, rebuilding dropped layers from their inputs
    for l in reversed(range(cfg.n_layers)):
        S = saved[l]
        if S is None:
            _, S = layer_forward(cfg, P, l, inputs[l], B, L, lengths, dropout)
        dh = layer_backward(cfg, P, l, S, dh, G)
        saved[l] = None

    # embedding backward
    if keep_e is not None:
        dh = dh * keep_e
    if cfg.pre_ln:
        demb = dh
    else:
        demb, G["emb_ln_g"], G["emb_ln_b"] = layernorm_bwd(dh, emb_saved, P["emb_ln_g"])
    dtok = np.zeros_like(P["tok_emb"])
    np.add.at(dtok, ids, demb)
    G["tok_emb"] = G["tok_emb"] + dtok
    dpos = np.zeros_like(P["pos_emb"])
    np.add.at(dpos, pos, demb)
    G["pos_emb"] = dpos

    if return_logits:
        return loss, G, logits
    return loss, G


def flops_per_step(cfg: Cfg, B: int, L: int, n_recomputed: int = 0, plan: int = None) -> Tuple[float, float]:
    """(useful, recompute) floating-point operations of one step, 2mnk per product.
    The recomputed layers are the first n_recomputed, or those whose bit is set in plan."""
    T = B * L
    H, V = cfg.hidden, cfg.vocab
    if plan is None:
        plan = (1 << n_recomputed) - 1
    attn = 4.0 * L * H * (0.5 if cfg.causal else 1.0)
    widths = [cfg.ffn_by_layer[l] if cfg.ffn_by_layer else cfg.ffn for l in range(cfg.n_layers)]
    layers = [8.0 * H * H + 4.0 * H * F + attn for F in widths]
    head = 2.0 * H * V + (2.0 * H * H if cfg.head else 0.0)
    useful = 3.0 * T * (sum(layers) + head)
    return useful, float(T) * sum(f for l, f in enumerate(layers) if (plan >> l) & 1)
