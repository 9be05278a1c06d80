"""Pins of the numeric oracle against things other than itself."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synthdata
from oracle import model as om

torch.set_num_threads(4)


def small_shape(**kw):
    base = dict(n_layers=2, hidden=16, n_heads=2, ffn=32, vocab=37, max_seq=8)
    base.update(kw)
    return synthdata.ModelShape(**base)


VARIANTS = [
    dict(),                                                        # post-LN, erf GELU, MLM head
    dict(causal=1, pre_ln=1, gelu_tanh=1, head=0),                 # GPT-2-shaped
    dict(causal=1),                                                # post-LN + causal mask
    dict(pre_ln=1, head=1),                                        # pre-LN with MLM head
]


def setup(shape, B, L, seed=3, perturb=True):
    params = synthdata.make_params(shape, seed, perturb=perturb)
    tokens, labels = synthdata.make_batch(shape, B, L, seed + 1)
    labels = labels.copy()
    if not shape.causal:
        labels[0, 0] = -1                                          # an ignored position
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    return cfg, params, tokens, labels


# ---------------------------------------------------------------- P1: finite differences
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("L", [3, 5])
def test_finite_differences(variant, L):
    shape = small_shape(**variant)
    cfg, params, tokens, labels = setup(shape, 2, L)
    params = {k: v.astype(np.float64) for k, v in params.items()}
    loss, G = om.train_step(cfg, params, tokens, labels)
    rng = np.random.default_rng(0)
    eps = 1e-5
    for name, p in params.items():
        assert name in G, name
        assert G[name].shape == p.shape
        idxs = [tuple(rng.integers(0, s) for s in p.shape) for _ in range(3)]
        if name == "tok_emb":                                       # rows that are certainly used
            idxs += [(int(tokens[0, 0]), 1), (int(tokens[1, L - 1]), 2)]
        if name == "pos_emb":
            idxs = [(int(rng.integers(0, L)), int(rng.integers(0, p.shape[1]))) for _ in range(3)]
        for idx in idxs:
            old = p[idx]
            p[idx] = old + eps
            lp, _ = om.train_step(cfg, params, tokens, labels)
            p[idx] = old - eps
            lm, _ = om.train_step(cfg, params, tokens, labels)
            p[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - G[name][idx]) <= 1e-6 * max(1.0, abs(fd)) + 2e-9, (name, idx, fd, G[name][idx])


# ------------------------------------------- independent derivation: torch library ops + autograd
def torch_loss(shape, params, tokens, labels):
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    B, L = tokens.shape
    H, nh = shape.hidden, shape.n_heads
    ids = torch.tensor(tokens.reshape(-1), dtype=torch.long)
    pos = torch.arange(L).repeat(B)
    gelu = (lambda x: F.gelu(x, approximate="tanh")) if shape.gelu_tanh else F.gelu
    ln = lambda x, g, b: F.layer_norm(x, (H,), P[g], P[b], shape.ln_eps)
    h = F.embedding(ids, P["tok_emb"]) + F.embedding(pos, P["pos_emb"])
    if not shape.pre_ln:
        h = ln(h, "emb_ln_g", "emb_ln_b")
    for l in range(shape.n_layers):
        p = f"layer{l}."
        a = ln(h, p + "ln1_g", p + "ln1_b") if shape.pre_ln else h
        qkv = F.linear(a, P[p + "wqkv"], P[p + "bqkv"]).reshape(B, L, 3, nh, H // nh)
        q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=bool(shape.causal))
        ctx = o.permute(0, 2, 1, 3).reshape(B * L, H)
        s1 = h + F.linear(ctx, P[p + "wo"], P[p + "bo"])
        if shape.pre_ln:
            u = s1
            f_in = ln(u, p + "ln2_g", p + "ln2_b")
        else:
            u = ln(s1, p + "ln1_g", p + "ln1_b")
            f_in = u
        s2 = u + F.linear(gelu(F.linear(f_in, P[p + "w1"], P[p + "b1"])), P[p + "w2"], P[p + "b2"])
        h = s2 if shape.pre_ln else ln(s2, p + "ln2_g", p + "ln2_b")
    if shape.pre_ln:
        h = ln(h, "final_ln_g", "final_ln_b")
    if shape.head:
        t = ln(gelu(F.linear(h, P["head.wt"], P["head.bt"])), "head.ln_g", "head.ln_b")
        logits = F.linear(t, P["tok_emb"], P["head.bdec"])
    else:
        logits = F.linear(h, P["tok_emb"])
    loss = F.cross_entropy(logits, torch.tensor(labels.reshape(-1), dtype=torch.long), ignore_index=-1)
    loss.backward()
    return float(loss.detach()), {k: v.grad.numpy() for k, v in P.items()}


@pytest.mark.parametrize("variant", VARIANTS)
def test_against_torch_autograd(variant):
    shape = small_shape(n_layers=3, hidden=24, n_heads=3, ffn=40, **variant)
    cfg, params, tokens, labels = setup(shape, 3, 7)
    loss, G = om.train_step(cfg, params, tokens, labels)
    tl, TG = torch_loss(shape, params, tokens, labels)
    assert abs(loss - tl) <= 1e-12 * abs(tl)
    for name in params:
        ref = TG[name]
        err = np.linalg.norm(G[name] - ref) / max(np.linalg.norm(ref), 1e-30)
        assert err < 1e-10, (name, err)


def test_fp32_build_matches_fp64():
    shape = small_shape()
    cfg, params, tokens, labels = setup(shape, 2, 8)
    l64, G64 = om.train_step(cfg, params, tokens, labels, dtype=np.float64)
    l32, G32 = om.train_step(cfg, params, tokens, labels, dtype=np.float32)
    assert abs(l64 - l32) < 1e-5 * abs(l64)
    for k in G64:
        assert np.linalg.norm(G64[k] - G32[k]) <= 1e-4 * np.linalg.norm(G64[k]) + 1e-9


# ---------------------------------------------------------------- P2: closed-form loss at init
@pytest.mark.parametrize("name,tol", [("tiny", 0.01)])
def test_initial_loss_closed_form(name, tol):
    wl = synthdata.WORKLOADS[name]
    shape = wl.shape
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    params = synthdata.make_params(shape, wl.seed)
    tokens, labels = synthdata.make_batch(shape, wl.batch, 32, 5)
    loss, _ = om.train_step(cfg, params, tokens, labels, dtype=np.float32)
    # unit-variance rows times N(0, 0.02^2) embeddings: logit variance 0.02^2 * H;
    # E[logsumexp] - E[picked logit] = ln V + variance / 2
    expect = math.log(shape.vocab) + 0.5 * 0.02 ** 2 * shape.hidden
    assert abs(loss - expect) < tol * expect


# ---------------------------------------------------------------- P3: invariants / special cases
def test_softmax_rows_and_l1_attention():
    rng = np.random.default_rng(1)
    q, k, v = (rng.standard_normal((2, 3, 6, 4)) for _ in range(3))
    o, p = om.attention_fwd(q, k, v, causal=0)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    o1, p1 = om.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1], causal=0)
    assert np.array_equal(p1, np.ones_like(p1))
    assert np.allclose(o1, v[:, :, :1])
    oc, pc = om.attention_fwd(q, k, v, causal=1)
    assert np.all(np.triu(pc[0, 0], k=1) == 0.0)
    assert np.allclose(oc[:, :, 0], v[:, :, 0])                    # first row attends to itself only


def test_layernorm_moments_and_gelu_values():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 64)) * 3 + 1
    y, _ = om.layernorm_fwd(x, np.ones(64), np.zeros(64), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-13) and np.allclose(y.var(-1), 1, atol=1e-12)
    xs = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    want = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in xs])
    assert np.allclose(om.gelu_fwd(xs, 0), want, atol=1e-15)
    # derivative of both forms against a central difference
    for form in (0, 1):
        fd = (om.gelu_fwd(xs + 1e-6, form) - om.gelu_fwd(xs - 1e-6, form)) / 2e-6
        assert np.allclose(om.gelu_grad(xs, form), fd, atol=1e-8)
    assert abs(om.gelu_fwd(np.array([1.0]), 1)[0] - 0.8411919906082768) < 1e-12   # tanh form at x=1


def test_cross_entropy_properties():
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((6, 11))
    labels = np.array([1, 4, -1, 0, 10, 3])
    loss, d = om.cross_entropy(logits, labels)
    assert np.allclose(d.sum(-1), 0, atol=1e-15)
    assert np.all(d[2] == 0)
    # uniform logits: loss is ln V
    l2, _ = om.cross_entropy(np.zeros((4, 11)), np.array([0, 1, 2, 3]))
    assert abs(l2 - math.log(11)) < 1e-14
    ref = F.cross_entropy(torch.tensor(logits), torch.tensor(labels), ignore_index=-1)
    assert abs(loss - float(ref)) < 1e-14


def test_bdec_gradient_sums_to_zero_and_causal_independence():
    shape = small_shape(causal=1)
    cfg, params, tokens, labels = setup(shape, 2, 6)
    loss, G, logits = om.train_step(cfg, params, tokens, labels, return_logits=True)
    assert abs(G["head.bdec"].sum()) < 1e-14
    t2 = tokens.copy()
    t2[:, 4:] = (t2[:, 4:] + 7) % shape.vocab                      # change the future
    _, _, logits2 = om.train_step(cfg, params, t2, labels, return_logits=True)
    lg = logits.reshape(2, 6, -1)
    lg2 = logits2.reshape(2, 6, -1)
    assert np.array_equal(lg[:, :4], lg2[:, :4])
    assert not np.allclose(lg[:, 4:], lg2[:, 4:])


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(4)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4096),
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], dtype=np.float32)])
    want = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(om.round_to_bf16(a), want)


# ---------------------------------------------------------------- P4: checkpointing leaves gradients unchanged
@pytest.mark.parametrize("variant", VARIANTS[:2])
def test_all_plans_bitwise_identical(variant):
    shape = small_shape(n_layers=4, **variant)
    cfg, params, tokens, labels = setup(shape, 2, 5)
    l0, G0 = om.train_step(cfg, params, tokens, labels, plan=0, dtype=np.float32)
    for plan in range(1, 16):
        l1, G1 = om.train_step(cfg, params, tokens, labels, plan=plan, dtype=np.float32)
        assert l1 == l0
        for k in G0:
            assert np.array_equal(G0[k], G1[k]), (plan, k)


# ---------------------------------------------------------------- padded batches
def _padded_case(causal):
    import synthdata
    shape = synthdata.ModelShape(2, 32, 2, 64, 50, 12, "fp32", causal=int(causal), pre_ln=int(causal),
                                 gelu_tanh=int(causal), head=0 if causal else 1)
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    params = {k: v.astype(np.float64) for k, v in synthdata.make_params(shape, 3, perturb=True).items()}
    tokens, labels = synthdata.make_batch(shape, 3, 9, 5)
    return shape, cfg, params, tokens, labels, np.array([9, 4, 6])


@pytest.mark.parametrize("causal", [False, True])
def test_padded_batch_equals_samples_run_alone(causal):
    """A batch padded to its longest sample with lengths given must be the samples run one by one
    at their own lengths: loss = label-count-weighted mean, gradients = label-count-weighted sum
    (a definition that involves no mask at all)."""
    shape, cfg, params, tokens, labels, lengths = _padded_case(causal)
    loss, G = om.train_step(cfg, params, tokens, labels, lengths=lengths)
    tot_n, tot_loss, tot_G = 0, 0.0, None
    for b, n in enumerate(lengths):
        t1, l1 = tokens[b:b + 1, :n], labels[b:b + 1, :n].copy()
        if causal:
            l1[0, n - 1] = -1                                       # the last real token has no successor
        nv = int((l1 >= 0).sum())
        ls, g = om.train_step(cfg, params, t1, l1)
        tot_n += nv; tot_loss += ls * nv
        tot_G = {k: v * nv for k, v in g.items()} if tot_G is None else {k: tot_G[k] + g[k] * nv for k in g}
    if causal:                                                      # same labels in the padded run
        lab2 = labels.copy()
        for b, n in enumerate(lengths):
            lab2[b, n - 1:] = -1
        loss, G = om.train_step(cfg, params, tokens, lab2, lengths=lengths)
    assert abs(loss - tot_loss / tot_n) < 1e-12
    for k in G:
        if k == "pos_emb":                                          # rows past a sample's length get nothing from it
            pass
        np.testing.assert_allclose(G[k], tot_G[k] / tot_n, rtol=1e-9, atol=1e-13, err_msg=k)


def test_padding_content_does_not_matter():
    shape, cfg, params, tokens, labels, lengths = _padded_case(False)
    loss, G = om.train_step(cfg, params, tokens, labels, lengths=lengths)
    t2 = tokens.copy()
    for b, n in enumerate(lengths):
        t2[b, n:] = (t2[b, n:] + 7) % shape.vocab
    loss2, G2 = om.train_step(cfg, params, t2, labels, lengths=lengths)
    assert loss == loss2
    for k in G:
        np.testing.assert_array_equal(G[k], G2[k])
    # full lengths are the unpadded definition
    loss3, G3 = om.train_step(cfg, params, tokens, labels, lengths=np.full(3, tokens.shape[1]))
    loss4, G4 = om.train_step(cfg, params, tokens, labels)
    assert loss3 == loss4 and all(np.array_equal(G3[k], G4[k]) for k in G3)


# ---------------------------------------------------------------- the FLOP count behind the throughput figures
class _CountingArray(np.ndarray):
    """ndarray that adds 2*m*n*k to a counter for every matrix product it takes part in."""
    flops = 0

    def __array_ufunc__(self, ufunc, method, *inputs, out=None, **kw):
        plain = tuple(i.view(np.ndarray) if isinstance(i, np.ndarray) else i for i in inputs)
        if out is not None:
            kw["out"] = tuple(o.view(np.ndarray) if isinstance(o, np.ndarray) else o for o in out)
        res = getattr(ufunc, method)(*plain, **kw)
        if ufunc is np.matmul and method == "__call__":
            a, b = plain
            _CountingArray.flops += 2 * int(np.prod(res.shape)) * a.shape[-1]
        if isinstance(res, tuple):
            return tuple(r.view(_CountingArray) if isinstance(r, np.ndarray) else r for r in res)
        return res.view(_CountingArray) if isinstance(res, np.ndarray) else res


def _counted_step(cfg, params, tokens, labels, plan):
    _CountingArray.flops = 0
    om.train_step(cfg, {k: v.astype(np.float64).view(_CountingArray) for k, v in params.items()}, tokens, labels, plan=plan)
    return _CountingArray.flops


@pytest.mark.parametrize("variant", [dict(), dict(pre_ln=1, head=0), dict(ffn_by_layer=(48, 32, 16), n_layers=3)])
def test_flops_per_step_equals_the_products_the_definition_performs(variant):
    """useful = every product of forward and backward at 2mnk; recompute = the products of the rebuilt
    layers' forwards: counted while the oracle runs, not retyped."""
    shape = small_shape(**variant)
    cfg, params, tokens, labels = setup(shape, 3, 7)
    base = _counted_step(cfg, params, tokens, labels, 0)
    assert base > 0
    useful, re0 = om.flops_per_step(cfg, 3, 7)
    assert re0 == 0.0 and useful == base
    for plan in range(1, 1 << shape.n_layers):
        u, re = om.flops_per_step(cfg, 3, 7, plan=plan)
        assert u == base and re == _counted_step(cfg, params, tokens, labels, plan) - base, plan
    assert om.flops_per_step(cfg, 3, 7, n_recomputed=2) == om.flops_per_step(cfg, 3, 7, plan=0b11)


def test_flops_per_step_worked_example_and_causal_half():
    """BERT-base at L = 200, B = 32: per token and layer 24H^2 + 4LH = 14.16 + 0.61 MFLOP, head
    2H^2 + 2HV = 1.18 + 46.88, forward 225.4, training 3 x forward = 676 MFLOP per token, 4.33 TFLOP
    per step; a rebuilt layer costs its forward again; a causal mask halves the attention term."""
    cfg = om.Cfg(12, 768, 12, 3072, 30522, 512)
    useful, re = om.flops_per_step(cfg, 32, 200, plan=0b101)
    T = 6400
    layer = 24 * 768 ** 2 + 4 * 200 * 768
    head = 2 * 768 ** 2 + 2 * 768 * 30522
    assert layer == 14_155_776 + 614_400 and head == 1_179_648 + 46_881_792
    assert useful == 3.0 * T * (12 * layer + head)
    assert abs(useful / T / 1e6 - 676.0) < 0.5 and abs(useful / 1e12 - 4.33) < 0.005
    assert re == 2.0 * T * layer
    causal = om.Cfg(12, 768, 12, 3072, 30522, 512, causal=1)
    uc, rc = om.flops_per_step(causal, 32, 200, plan=0b1)
    assert useful - uc == 3.0 * T * 12 * (2 * 200 * 768)
    assert rc == T * (24 * 768 ** 2 + 2 * 200 * 768)
    lm = om.Cfg(12, 768, 12, 3072, 30522, 512, head=0)
    assert useful - om.flops_per_step(lm, 32, 200)[0] == 3.0 * T * 2 * 768 ** 2
