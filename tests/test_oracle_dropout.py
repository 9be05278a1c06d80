"""Pins of the oracle's counter-based dropout: the generator against its published known-answer
vectors, the masks against what a dropout mask must be, and the gradients with dropout against
finite differences and against torch autograd given the same masks."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synthdata
from oracle import model as om
from oracle import philox as ph
from test_oracle_model import VARIANTS, setup, small_shape

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_kat():
    out = []
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.strip() and not line.startswith("#"):
            v = [int(w, 16) for w in line.split()]
            out.append((v[:4], v[4:6], v[6:]))
    return out


@pytest.mark.parametrize("ctr,key,want", read_kat())
def test_generator_known_answers(ctr, key, want):
    assert [int(w) for w in ph.philox4x32_10(*ctr, *key)] == want


def test_generator_is_vectorised_consistently():
    kat = read_kat()
    c = np.array([k[0] for k in kat], dtype=np.uint64)
    for (ctr, key, want) in kat:                      # one key at a time, all counters at once
        got = ph.philox4x32_10(c[:, 0], c[:, 1], c[:, 2], c[:, 3], *key)
        i = [k[0] for k in kat].index(ctr)
        assert [int(w[i]) for w in got] == want


def test_four_neighbouring_elements_share_one_block():
    # elements 4b .. 4b+3 read words 0..3 of block b, whose number fills counter words 0 and 1;
    # site, step and the two halves of the seed fill the rest
    seed, site, step = 0x299f31d0a4093822, 0x13198a2e, 0x03707344
    b = 0x05a308d3243f6a88
    idx = np.array([4 * b + j for j in range(4)], dtype=np.uint64)
    want = ph.philox4x32_10(0x243f6a88, 0x05a308d3, site, step, 0xa4093822, 0x299f31d0)
    assert [int(w) for w in ph.words_at(idx, seed, site, step)] == [int(w) for w in want]
    assert [int(w) for w in ph.words_at(np.arange(4, dtype=np.uint64), 0, 0, 0)] == read_kat()[0][2]
    assert [int(w) for w in ph.words_at(np.array([2, 1], dtype=np.uint64), 0, 0, 0)] == [read_kat()[0][2][2], read_kat()[0][2][1]]


def test_threshold():
    assert ph.threshold(0.0) == 0
    assert ph.threshold(0.5) == 1 << 31
    assert ph.threshold(np.float32(0.1)) == int(np.floor(float(np.float32(0.1)) * 2.0 ** 32 + 0.5))
    assert ph.threshold(0.99999999) == 0xFFFFFFFF                     # float32 rounds this to 1: clamp


@pytest.mark.parametrize("p", [0.1, 0.5])
def test_mask_statistics(p):
    n = 1 << 20
    idx = np.arange(n, dtype=np.uint64)
    k = ph.keep_scale(idx, p, seed=7, site=ph.site_ffn_out(3), step=11)
    kept = k > 0
    sigma = np.sqrt(p * (1 - p) / n)
    assert abs(kept.mean() - (1 - p)) < 4.5 * sigma
    assert np.allclose(k[kept], 1.0 / (1.0 - float(np.float32(p))), rtol=0, atol=1e-15)
    assert abs(k.mean() - 1.0) < 6 * sigma / (1 - p)                  # the expectation is preserved
    w = ph.words_at(idx, 7, ph.site_ffn_out(3), 11)
    for bit in range(32):                                             # every bit of the word is fair
        assert abs(((w >> np.uint32(bit)) & np.uint32(1)).mean() - 0.5) < 4.5 * 0.5 / np.sqrt(n)
    # neighbours are uncorrelated
    a, b = kept[:-1].astype(float), kept[1:].astype(float)
    assert abs(np.corrcoef(a, b)[0, 1]) < 5 / np.sqrt(n)


def test_masks_differ_between_sites_steps_and_seeds():
    idx = np.arange(1 << 16, dtype=np.uint64)
    p = 0.3
    base = ph.keep_scale(idx, p, 1, ph.site_attn_out(0), 5) > 0
    same = ph.keep_scale(idx, p, 1, ph.site_attn_out(0), 5) > 0
    assert np.array_equal(base, same)                                 # a replay gives the same mask
    agree = (1 - p) ** 2 + p ** 2
    for other in (ph.keep_scale(idx, p, 1, ph.site_ffn_out(0), 5), ph.keep_scale(idx, p, 1, ph.site_attn_out(1), 5),
                  ph.keep_scale(idx, p, 1, ph.site_attn_out(0), 6), ph.keep_scale(idx, p, 2, ph.site_attn_out(0), 5),
                  ph.keep_scale(idx, p, 1 + (1 << 32), ph.site_attn_out(0), 5)):
        assert abs(((other > 0) == base).mean() - agree) < 0.01
    sites = [ph.SITE_EMBED] + [f(l) for l in range(64) for f in (ph.site_attn_prob, ph.site_attn_out, ph.site_ffn_out)]
    assert len(set(sites)) == len(sites)


def test_attention_rows_are_padded_to_four_keys():
    for L in (5, 8):
        idx = ph.attn_index(2, 3, L)
        assert idx.shape == (2, 3, L, L)
        assert len(np.unique(idx)) == idx.size
        assert (idx[..., 0] % 4 == 0).all()                           # every row starts a block
        assert (idx[..., 1:] - idx[..., :-1] == 1).all()


# ---------------------------------------------------------------- the model with dropout
DROP = om.Dropout(p_hidden=0.25, p_attn=0.2, seed=0x1234567890ABCDEF, step=3)


def test_zero_probability_changes_nothing():
    shape = small_shape()
    cfg, params, tokens, labels = setup(shape, 2, 5)
    l0, G0 = om.train_step(cfg, params, tokens, labels)
    l1, G1 = om.train_step(cfg, params, tokens, labels, dropout=om.Dropout(0.0, 0.0, 9, 9))
    assert l0 == l1 and all(np.array_equal(G0[k], G1[k]) for k in G0)
    l2, _ = om.train_step(cfg, params, tokens, labels, dropout=DROP)
    assert l2 != l0
    l3, _ = om.train_step(cfg, params, tokens, labels, dropout=om.Dropout(0.25, 0.2, DROP.seed, 4))
    assert l3 != l2                                                   # another iteration, other masks


@pytest.mark.parametrize("variant", VARIANTS[:2])
def test_finite_differences_with_dropout(variant):
    """The masks are a function of (seed, step, site, element) only, so the loss stays a smooth
    function of the parameters and central differences apply."""
    shape = small_shape(**variant)
    cfg, params, tokens, labels = setup(shape, 2, 5)
    params = {k: v.astype(np.float64) for k, v in params.items()}
    loss, G = om.train_step(cfg, params, tokens, labels, dropout=DROP)
    rng = np.random.default_rng(1)
    eps = 1e-5
    for name, p in params.items():
        idxs = [tuple(rng.integers(0, s) for s in p.shape) for _ in range(2)]
        if name == "tok_emb":
            idxs += [(int(tokens[0, 0]), 1)]
        if name == "pos_emb":
            idxs = [(int(rng.integers(0, 5)), int(rng.integers(0, p.shape[1]))) for _ in range(2)]
        for idx in idxs:
            old = p[idx]
            p[idx] = old + eps
            lp, _ = om.train_step(cfg, params, tokens, labels, dropout=DROP)
            p[idx] = old - eps
            lm, _ = om.train_step(cfg, params, tokens, labels, dropout=DROP)
            p[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - G[name][idx]) <= 1e-6 * max(1.0, abs(fd)) + 2e-9, (name, idx, fd, G[name][idx])


def torch_loss_with_masks(shape, params, tokens, labels, drop):
    """The same model written with torch ops and differentiated by autograd; dropout enters as
    given multipliers (torch's own dropout draws from another generator)."""
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    B, L = tokens.shape
    T, H, nh = B * L, shape.hidden, shape.n_heads
    hid = lambda site: torch.tensor(ph.keep_scale(ph.hidden_index(T, H), drop.p_hidden, drop.seed, site, drop.step))
    ids = torch.tensor(tokens.reshape(-1), dtype=torch.long)
    pos = torch.arange(L).repeat(B)
    gelu = (lambda x: F.gelu(x, approximate="tanh")) if shape.gelu_tanh else F.gelu
    ln = lambda x, g, b: F.layer_norm(x, (H,), P[g], P[b], shape.ln_eps)
    h = F.embedding(ids, P["tok_emb"]) + F.embedding(pos, P["pos_emb"])
    if not shape.pre_ln:
        h = ln(h, "emb_ln_g", "emb_ln_b")
    h = h * hid(ph.SITE_EMBED)
    for l in range(shape.n_layers):
        p = f"layer{l}."
        a = ln(h, p + "ln1_g", p + "ln1_b") if shape.pre_ln else h
        qkv = F.linear(a, P[p + "wqkv"], P[p + "bqkv"]).reshape(B, L, 3, nh, H // nh)
        q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))
        s = q @ k.transpose(-1, -2) / (H // nh) ** 0.5
        if shape.causal:
            s = s.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
        keep_p = torch.tensor(ph.keep_scale(ph.attn_index(B, nh, L), drop.p_attn, drop.seed, ph.site_attn_prob(l), drop.step))
        o = (torch.softmax(s, -1) * keep_p) @ v
        ctx = o.permute(0, 2, 1, 3).reshape(T, H)
        s1 = h + F.linear(ctx, P[p + "wo"], P[p + "bo"]) * hid(ph.site_attn_out(l))
        if shape.pre_ln:
            u = s1
            f_in = ln(u, p + "ln2_g", p + "ln2_b")
        else:
            u = ln(s1, p + "ln1_g", p + "ln1_b")
            f_in = u
        s2 = u + F.linear(gelu(F.linear(f_in, P[p + "w1"], P[p + "b1"])), P[p + "w2"], P[p + "b2"]) * hid(ph.site_ffn_out(l))
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
def test_against_torch_autograd_with_the_same_masks(variant):
    shape = small_shape(n_layers=3, hidden=24, n_heads=3, ffn=40, **variant)
    cfg, params, tokens, labels = setup(shape, 3, 7)
    loss, G = om.train_step(cfg, params, tokens, labels, dropout=DROP)
    tl, TG = torch_loss_with_masks(shape, params, tokens, labels, DROP)
    assert abs(loss - tl) <= 1e-12 * abs(tl)
    for name in params:
        err = np.linalg.norm(G[name] - TG[name]) / max(np.linalg.norm(TG[name]), 1e-30)
        assert err < 1e-10, (name, err)


@pytest.mark.parametrize("variant", VARIANTS[:2])
def test_recomputed_layers_replay_their_masks(variant):
    shape = small_shape(n_layers=3, **variant)
    cfg, params, tokens, labels = setup(shape, 2, 6)
    l0, G0 = om.train_step(cfg, params, tokens, labels, dropout=DROP)
    for plan in range(1, 8):
        l1, G1 = om.train_step(cfg, params, tokens, labels, plan=plan, dropout=DROP)
        assert l1 == l0
        for k in G0:
            assert np.array_equal(G0[k], G1[k]), (plan, k)


def test_dropout_with_padded_batch_equals_masks_applied_to_the_padded_run():
    """Padding and dropout are independent: masks are indexed by position in the padded tensor."""
    shape = small_shape()
    cfg, params, tokens, labels = setup(shape, 3, 8)
    lengths = np.array([8, 3, 5])
    l0, G0 = om.train_step(cfg, params, tokens, labels, lengths=lengths, dropout=DROP)
    t2 = tokens.copy()
    for b, n in enumerate(lengths):
        t2[b, n:] = 1
    l1, G1 = om.train_step(cfg, params, t2, labels, lengths=lengths, dropout=DROP)
    assert l0 == l1
    for k in G0:
        if k not in ("tok_emb",):
            assert np.array_equal(G0[k], G1[k]), k
