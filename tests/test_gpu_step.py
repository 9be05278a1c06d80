"""Whole-step parity of the HIP path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import synthdata
import paper_2209_02478_amd as mi
from oracle import model as om
from oracle import planner as op
from gpu_util import rel_l2

pytestmark = pytest.mark.gpu

MiB = 1 << 20


def oracle_step(shape, params, tokens, labels, dtype=np.float64, lengths=None):
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    if shape.dtype == "bf16":
        params = {k: om.round_to_bf16(v) for k, v in params.items()}
    return om.train_step(cfg, params, tokens, labels, dtype=dtype, lengths=lengths)


def oracle_step_dropout(shape, params, tokens, labels, dropout, lengths=None):
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    if shape.dtype == "bf16":
        params = {k: om.round_to_bf16(v) for k, v in params.items()}
    return om.train_step(cfg, params, tokens, labels, lengths=lengths, dropout=dropout)


def check_against_oracle(shape, m, params, tokens, labels, loss_tol, grad_tol, oracle_dtype=np.float64, lengths=None):
    loss, peak, plan = m.train_step(tokens, labels, lengths=lengths)
    G = m.grads()
    ref_loss, RG = oracle_step(shape, params, tokens, labels, oracle_dtype, lengths)
    assert abs(loss - ref_loss) <= loss_tol * abs(ref_loss), (loss, ref_loss)
    worst = check_grads(G, RG, grad_tol)
    return loss, peak, plan, worst


def check_grads(G, RG, grad_tol):
    """Every gradient tensor: relative L2 error within grad_tol, and no single element further from
    the oracle's than MAX_ABS_FACTOR * grad_tol times the tensor's largest magnitude (a tensor norm
    alone would let a few wrong rows of an embedding gradient through)."""
    worst, worst_abs = ("", 0.0), ("", 0.0)
    for k, ref in RG.items():
        e = rel_l2(G[k], ref)
        a = float(np.max(np.abs(np.asarray(G[k], dtype=np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))
        if e > worst[1]:
            worst = (k, e)
        if a > worst_abs[1]:
            worst_abs = (k, a)
        assert e <= grad_tol, (k, e)
        assert a <= MAX_ABS_FACTOR * grad_tol, (k, a)
    print("worst rel-L2", worst, "worst max-abs / max|ref|", worst_abs)
    return worst


MAX_ABS_FACTOR = 4.0


SMALL = {
    "fp32_postln": synthdata.ModelShape(2, 64, 2, 256, 1000, 64, "fp32"),
    "fp32_preln_causal": synthdata.ModelShape(3, 64, 2, 128, 300, 48, "fp32", causal=1, pre_ln=1, gelu_tanh=1, head=0),
    "fp32_preln_head": synthdata.ModelShape(2, 128, 2, 256, 200, 40, "fp32", pre_ln=1, head=1),
    "bf16_postln": synthdata.ModelShape(3, 128, 2, 512, 1000, 96, "bf16"),
    "bf16_preln_causal": synthdata.ModelShape(2, 256, 4, 512, 777, 80, "bf16", causal=1, pre_ln=1, gelu_tanh=1, head=0),
    # layers of different feed-forward widths
    "fp32_stages": synthdata.ModelShape(3, 64, 2, 256, 500, 48, "fp32", ffn_by_layer=(320, 100, 36)),
    "bf16_stages": synthdata.ModelShape(3, 128, 2, 512, 1000, 96, "bf16", pre_ln=1, ffn_by_layer=(768, 264, 128)),
}


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("B,L", [(4, 33), (2, 7)])
def test_step_parity_small_models(name, B, L):
    shape = SMALL[name]
    params = synthdata.make_params(shape, 11, perturb=True)
    tokens, labels = synthdata.make_batch(shape, B, L, 12)
    if not shape.causal:
        labels = labels.copy(); labels[0, 1] = -1
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    m.force_plan(0)
    fp32 = shape.dtype == "fp32"
    check_against_oracle(shape, m, params, tokens, labels, 1e-4 if fp32 else 1e-2, 1e-3 if fp32 else 2e-2)
    m.close()


@pytest.mark.parametrize("name", ["fp32_postln", "bf16_postln", "bf16_preln_causal", "fp32_stages", "bf16_stages"])
def test_checkpointed_gradients_bit_identical(name):
    shape = SMALL[name]
    n = shape.n_layers
    params = synthdata.make_params(shape, 21, perturb=True)
    tokens, labels = synthdata.make_batch(shape, 4, 40, 22)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    m.force_plan(0)
    loss0, peak0, _ = m.train_step(tokens, labels)
    G0 = m.grads()
    peaks = {0: peak0}
    for plan in range(1, 1 << n):
        m.force_plan(plan)
        loss, peak, got = m.train_step(tokens, labels)
        assert got == plan and loss == loss0
        peaks[plan] = peak
        G = m.grads()
        for k in G0:
            assert np.array_equal(G0[k], G[k]), (plan, k)
    assert peaks[(1 << n) - 1] == min(peaks.values()) < peak0
    m.close()


@pytest.mark.parametrize("name,cost_aware", [("tiny", 0), ("tiny_stages", 0), ("tiny_stages", 1)])
def test_tiny_workload_every_step(name, cost_aware):
    """The small fp32 configurations end to end: sheltered then responsive steps under the
    budget, every step checked against the oracle and the oracle planner (with the measured
    forward times of the sheltered steps when the selection is cost-aware)."""
    wl = synthdata.WORKLOADS[name]
    shape, B, n = wl.shape, wl.batch, wl.shape.n_layers
    d = synthdata.shape_dict(shape)
    cal = mi.Mimose(d, 0, device=None)
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, shape.max_seq)
    cal.close()
    budget = int(wl.budget_frac * peak0)
    params = synthdata.make_params(shape, wl.seed)
    m = mi.Mimose(d, budget, cost_aware=cost_aware)
    m.load_params(params)
    ref = op.Planner(n, budget, guard=4096, cost_aware=bool(cost_aware))
    lens = synthdata.seq_lengths(wl.length_recipe, wl.steps, wl.seed)
    plans = []
    for i, L in enumerate(lens):
        tokens, labels = synthdata.make_batch(shape, B, L, synthdata.step_seed(wl.seed, i))
        sheltered = ref.sheltered()
        loss, peak, plan, worst = check_against_oracle(shape, m, params, tokens, labels, 1e-4, 1e-3)
        assert peak <= budget
        mem = m.step_memory()
        c = op.Components(F=mem["F"], e=mem["e"], g=mem["g"], a=mem["a"], b=mem["b"], w=mem["w"])
        assert peak == op.simulate_peak(c, plan)
        x = B * L
        if sheltered:
            assert plan == (1 << n) - 1
            for l in range(n):
                ref.feed(x, op.Q_A, l, c.a[l]); ref.feed(x, op.Q_B, l, c.b[l]); ref.feed(x, op.Q_W, l, c.w[l])
            ref.feed(x, op.Q_E, -1, c.e); ref.feed(x, op.Q_G, -1, c.g); ref.feed(x, op.Q_F, -1, c.F)
            times = m.layer_times()
            assert all(t > 0 for t in times)
            for l in range(n):
                ref.feed(x, op.Q_T, l, times[l])
            ref.end_sheltered_step(x)
        else:
            assert plan == ref.query(x).plan
        plans.append(plan)
    st = m.stats()
    assert st["steps"] == wl.steps and st["sheltered_steps"] == 10
    assert st["cache_hits"] == ref.hits and st["cache_misses"] == ref.misses
    m.close()


@pytest.mark.parametrize("name", ["fp32_postln", "bf16_preln_causal", "bf16_postln"])
def test_degenerate_batches(name):
    """One token; the longest admissible sequence; a batch in which no position is scored."""
    shape = SMALL[name]
    fp32 = shape.dtype == "fp32"
    params = synthdata.make_params(shape, 21, perturb=True)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    m.force_plan(1)
    for B, L in ((1, 1), (1, 2), (3, shape.max_seq)):
        tokens, labels = synthdata.make_batch(shape, B, L, 30 + L)
        if shape.causal and L == 1:
            continue                                   # a causal batch of length 1 has no scored position: below
        check_against_oracle(shape, m, params, tokens, labels, 1e-4 if fp32 else 1e-2, 1e-3 if fp32 else 2e-2)
    tokens, labels = synthdata.make_batch(shape, 2, 5, 44)
    labels = np.full_like(labels, -1)
    loss, _, _ = m.train_step(tokens, labels)
    assert loss == 0.0
    for k, g in m.grads().items():
        assert not np.any(g), k
    if shape.causal:
        tokens, labels = synthdata.make_batch(shape, 2, 1, 45)
        loss, _, _ = m.train_step(tokens, labels)
        assert loss == 0.0
    with pytest.raises(mi.MimoseError) as e:
        m.train_step(*synthdata.make_batch(shape, 1, shape.max_seq + 1, 46))      # longer than the position table
    assert e.value.code == mi.MIMOSE_ERR_INVALID_ARG
    m.close()


@pytest.mark.parametrize("name", list(SMALL))
def test_padded_batches(name):
    """Samples of their own lengths padded to the longest (Section 3.1): parity with the oracle,
    the same bits under every plan, nothing depends on what the padding holds, memory and plan
    are those of the unpadded call at the same B and L, and lengths == L is the unpadded step."""
    shape = SMALL[name]
    fp32 = shape.dtype == "fp32"
    n = shape.n_layers
    params = synthdata.make_params(shape, 51, perturb=True)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    m.force_plan(0)
    for lengths in ([33, 2, 17, 32], [7, 7, 1], [shape.max_seq, 3]):
        tokens, labels, lens = synthdata.make_padded_batch(shape, lengths, 60 + len(lengths))
        if not shape.causal:
            labels[0, 0] = -1
        loss0, peak0, _, _ = check_against_oracle(shape, m, params, tokens, labels, 1e-4 if fp32 else 1e-2,
                                                  1e-3 if fp32 else 2e-2, lengths=lens)
        G0 = m.grads()
        m.force_plan((1 << n) - 1)
        loss1, peak1, plan1 = m.train_step(tokens, labels, lengths=lens)
        assert loss1 == loss0 and plan1 == (1 << n) - 1 and peak1 < peak0
        G1 = m.grads()
        m.force_plan(0)
        # other ids and labels in the padding: the same bits, except that the padding ids' own
        # embedding rows are no longer touched (they got exact zeros before)
        t2, l2 = tokens.copy(), labels.copy()
        for b, k in enumerate(lens):
            t2[b, k:] = (7 * b + 3) % shape.vocab
            l2[b, k:] = 5
        loss2, peak2, _ = m.train_step(t2, l2, lengths=lens)
        G2 = m.grads()
        assert loss2 == loss0 and peak2 == peak0
        for k in G0:
            assert np.array_equal(G0[k], G1[k]), k
            assert np.array_equal(G0[k], G2[k]), k
        _, peak3, _ = m.train_step(tokens, labels)                   # unpadded call, same B and L
        assert peak3 == peak0
    tokens, labels = synthdata.make_batch(shape, 3, 20, 70)
    la, _, _ = m.train_step(tokens, labels)
    Ga = m.grads()
    lb, _, _ = m.train_step(tokens, labels, lengths=np.full(3, 20))
    Gb = m.grads()
    assert la == lb
    for k in Ga:
        assert np.array_equal(Ga[k], Gb[k]), k
    for bad in ([0, 20, 20], [21, 20, 20]):
        with pytest.raises(mi.MimoseError) as e:
            m.train_step(tokens, labels, lengths=np.array(bad))
        assert e.value.code == mi.MIMOSE_ERR_INVALID_ARG
    m.close()


@pytest.mark.parametrize("name", list(SMALL))
def test_dropout_parity_and_replay(name):
    """Dropout with counter-based masks: parity with the oracle given (p, seed, iteration), the
    same bits whether a layer's forward ran once or was rebuilt, other masks in the next
    iteration, and the plain step again once it is switched off."""
    shape = SMALL[name]
    fp32 = shape.dtype == "fp32"
    n = shape.n_layers
    p, pa = float(np.float32(0.15)), float(np.float32(0.1))
    seed = 0xC0FFEE1234567
    params = synthdata.make_params(shape, 81, perturb=True)
    tokens, labels = synthdata.make_batch(shape, 4, 33, 82)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    m.force_plan(0)
    plain_loss, plain_peak, _ = m.train_step(tokens, labels)
    plain_G = m.grads()

    def run(step, plan):
        m.set_dropout(p, pa, seed, step)
        m.force_plan(plan)
        loss, peak, _ = m.train_step(tokens, labels)
        return loss, peak, m.grads()

    loss0, peak0, G0 = run(5, 0)
    ref_loss, RG = oracle_step_dropout(shape, params, tokens, labels, om.Dropout(p, pa, seed, 5))
    assert abs(loss0 - ref_loss) <= (1e-4 if fp32 else 1e-2) * abs(ref_loss)
    for k, ref in RG.items():
        assert rel_l2(G0[k], ref) <= (1e-3 if fp32 else 2e-2), k
    assert loss0 != plain_loss and peak0 >= plain_peak           # masked gradient copies live in the backward
    for plan in range(1, 1 << n):
        loss, _, G = run(5, plan)
        assert loss == loss0
        for k in G0:
            assert np.array_equal(G0[k], G[k]), (plan, k)
    # the library counts iterations itself: the step after 5 is 6
    m.set_dropout(p, pa, seed, 5)
    m.force_plan(0)
    m.train_step(tokens, labels)
    loss6, _, _ = m.train_step(tokens, labels)
    ref6, _ = oracle_step_dropout(shape, params, tokens, labels, om.Dropout(p, pa, seed, 6))
    assert loss6 != loss0 and abs(loss6 - ref6) <= (1e-4 if fp32 else 1e-2) * abs(ref6)
    # padded batch and dropout together
    tk, lb, lens = synthdata.make_padded_batch(shape, [20, 7, 13], 83)
    m.set_dropout(p, pa, seed, 9)
    lossp, _, _ = m.train_step(tk, lb, lengths=lens)
    refp, RGp = oracle_step_dropout(shape, params, tk, lb, om.Dropout(p, pa, seed, 9), lens)
    assert abs(lossp - refp) <= (1e-4 if fp32 else 1e-2) * abs(refp)
    Gp = m.grads()
    for k, ref in RGp.items():
        assert rel_l2(Gp[k], ref) <= (1e-3 if fp32 else 2e-2), k
    # off again: the plain step, bit for bit
    m.set_dropout(0.0, 0.0, 0, 0)
    loss, peak, _ = m.train_step(tokens, labels)
    assert loss == plain_loss and peak == plain_peak
    for k, g in m.grads().items():
        assert np.array_equal(g, plain_G[k]), k
    with pytest.raises(mi.MimoseError):
        m.set_dropout(1.0, 0.0, 0, 0)
    with pytest.raises(mi.MimoseError):
        m.set_dropout(0.1, -0.1, 0, 0)
    m.close()


@pytest.mark.parametrize("name", ["fp32_postln", "bf16_postln", "bf16_preln_causal", "bf16_stages"])
def test_stream_layout_does_not_change_the_bits(name):
    """With per-kernel timing on, every kernel runs on the caller's stream over the whole batch;
    without it the forward runs as two halves of the batch on two streams and the weight
    gradients on the second one.  Same loss and gradients, bit for bit, also for an odd batch
    and for a padded one."""
    shape = SMALL[name]
    params = synthdata.make_params(shape, 91, perturb=True)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
    m.load_params(params)
    for B, L, plan in ((4, 33, 0), (5, 40, 0b101 & ((1 << shape.n_layers) - 1)), (2, 7, 1), (1, 16, 0)):
        tokens, labels = synthdata.make_batch(shape, B, L, 92 + B)
        m.force_plan(plan)
        mi.mimose_profile_enable(m.ctx, 1)
        loss0, _, _ = m.train_step(tokens, labels)
        G0 = m.grads()
        mi.mimose_profile_enable(m.ctx, 0)
        loss1, _, _ = m.train_step(tokens, labels)
        G1 = m.grads()
        assert loss0 == loss1
        for k in G0:
            assert np.array_equal(G0[k], G1[k]), (B, L, k)
    tk, lb, lens = synthdata.make_padded_batch(shape, [20, 7, 13], 93)
    m.force_plan(0)
    mi.mimose_profile_enable(m.ctx, 1)
    loss0, _, _ = m.train_step(tk, lb, lengths=lens)
    G0 = m.grads()
    mi.mimose_profile_enable(m.ctx, 0)
    loss1, _, _ = m.train_step(tk, lb, lengths=lens)
    G1 = m.grads()
    assert loss0 == loss1
    for k in G0:
        assert np.array_equal(G0[k], G1[k]), k
    m.close()


def test_static_plan_mode_same_gradients_more_recompute():
    """One plan for the longest input (the static planner of Section 3.2) against the input-aware
    planner on the small workload: bit-identical losses and gradients on every step, never fewer
    recomputed layers, both under the budget."""
    wl = synthdata.WORKLOADS["tiny"]
    shape, B, n = wl.shape, wl.batch, wl.shape.n_layers
    d = synthdata.shape_dict(shape)
    cal = mi.Mimose(d, 0, device=None)
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, shape.max_seq)
    cal.close()
    budget = int(wl.budget_frac * peak0)
    params = synthdata.make_params(shape, wl.seed)
    aware, static = mi.Mimose(d, budget), mi.Mimose(d, budget)
    static.set_plan_mode("static_max")
    for m in (aware, static):
        m.load_params(params)
    lens = synthdata.seq_lengths(wl.length_recipe, wl.steps, wl.seed)
    fewer = 0
    for i, L in enumerate(lens):
        tokens, labels = synthdata.make_batch(shape, B, L, synthdata.step_seed(wl.seed, i))
        la, pa, plan_a = aware.train_step(tokens, labels)
        ls, ps, plan_s = static.train_step(tokens, labels)
        assert la == ls and pa <= budget and ps <= budget
        ga, gs = aware.grads(), static.grads()
        for k in ga:
            assert np.array_equal(ga[k], gs[k]), k
        assert bin(plan_a).count("1") <= bin(plan_s).count("1")
        fewer += bin(plan_a).count("1") < bin(plan_s).count("1")
    assert fewer > 0
    assert static.stats()["cache_misses"] == 1
    aware.close(); static.close()


def test_bert_base_shape_step():
    """BERT-base shape, bf16, full batch of 32 at the shortest length: parity with the oracle
    (float32 build, bf16-rounded weights)."""
    wl = synthdata.WORKLOADS["bert_base"]
    shape = wl.shape
    params = synthdata.make_params(shape, wl.seed)
    tokens, labels = synthdata.make_batch(shape, wl.batch, 64, 5)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=4096 * MiB)
    m.load_params(params)
    m.force_plan(0)
    loss, peak, plan, worst = check_against_oracle(shape, m, params, tokens, labels, 1e-2, 2e-2, np.float32)
    print("bert_base L=64: loss", loss, "worst grad", worst)
    # same batch with half the layers dropped: identical bits
    G0 = m.grads()
    m.force_plan(0b010101010101)
    loss2, peak2, _ = m.train_step(tokens, labels)
    assert loss2 == loss and peak2 < peak
    G1 = m.grads()
    for k in G0:
        assert np.array_equal(G0[k], G1[k]), k
    m.close()


def test_bert_base_shape_padded_with_dropout():
    """BERT-base shape, full batch of 32 padded to L = 64 with per-sample lengths, dropout 0.1 on
    every site, half the layers rebuilt: parity with the oracle (float32 build, bf16-rounded
    weights) and the same bits as the run that keeps every layer."""
    wl = synthdata.WORKLOADS["bert_base"]
    shape = wl.shape
    params = synthdata.make_params(shape, wl.seed)
    rng = np.random.default_rng(7)
    lengths = [64] + [int(v) for v in rng.integers(8, 65, wl.batch - 1)]
    tokens, labels, lens = synthdata.make_padded_batch(shape, lengths, 6)
    p = float(np.float32(0.1))
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=4096 * MiB)
    m.load_params(params)
    m.set_dropout(p, p, 2024, 3)
    m.force_plan(0b101010101010)
    loss, peak, _ = m.train_step(tokens, labels, lengths=lens)
    G = m.grads()
    ref_loss, RG = oracle_step_dropout(shape, params, tokens, labels, om.Dropout(p, p, 2024, 3), lens)
    assert abs(loss - ref_loss) <= 1e-2 * abs(ref_loss), (loss, ref_loss)
    worst = max((rel_l2(G[k], ref), k) for k, ref in RG.items())
    print("bert_base padded + dropout: loss", loss, ref_loss, "worst grad", worst)
    assert worst[0] <= 2e-2, worst
    check_grads(G, RG, 2e-2)
    m.set_dropout(p, p, 2024, 3)
    m.force_plan(0)
    loss0, peak0, _ = m.train_step(tokens, labels, lengths=lens)
    assert loss0 == loss and peak0 > peak
    for k, g in m.grads().items():
        assert np.array_equal(g, G[k]), k
    m.close()


def test_bert_stages_shape_step():
    """The stack with three feed-forward widths at full size (batch 32, L = 64): parity with the oracle."""
    wl = synthdata.WORKLOADS["bert_stages"]
    shape = wl.shape
    params = synthdata.make_params(shape, wl.seed)
    tokens, labels = synthdata.make_batch(shape, wl.batch, 64, 5)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=4096 * MiB)
    m.load_params(params)
    m.force_plan(0b000011110000)
    loss, peak, plan, worst = check_against_oracle(shape, m, params, tokens, labels, 1e-2, 2e-2, np.float32)
    print("bert_stages L=64: loss", loss, "worst grad", worst)
    m.close()


def test_bert_base_full_length_under_budget():
    """Launch configuration of the benchmark at the longest length (B=32, L=512): the planner
    keeps the measured peak under 60 % of the no-checkpoint peak, the loss sits at its
    closed-form initial value and checkpointed gradients equal the unconstrained ones bit for bit."""
    wl = synthdata.WORKLOADS["bert_base"]
    shape, B = wl.shape, wl.batch
    d = synthdata.shape_dict(shape)
    cal = mi.Mimose(d, 0, device=None)
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, 512)
    cal.close()
    budget = int(wl.budget_frac * peak0)
    params = synthdata.make_params(shape, wl.seed)
    m = mi.Mimose(d, budget, arena_bytes=peak0 + MiB)
    m.load_params(params)
    lens = [64, 128, 200, 264, 320, 400, 448, 512, 96, 160]
    for i, L in enumerate(lens):                          # sheltered phase
        tokens, labels = synthdata.make_batch(shape, B, L, 100 + i)
        loss, peak, plan = m.train_step(tokens, labels)
        assert plan == (1 << 12) - 1 and peak <= budget
    tokens, labels = synthdata.make_batch(shape, B, 512, 999)
    loss, peak, plan = m.train_step(tokens, labels)
    assert plan != 0 and peak <= budget
    expect = np.log(shape.vocab) + 0.5 * 0.02 ** 2 * shape.hidden
    assert abs(loss - expect) < 0.02 * expect
    G1 = m.grads()
    short = m.train_step(*synthdata.make_batch(shape, B, 64, 998))
    assert short[2] == 0 and short[1] <= budget
    m.close()
    big = mi.Mimose(d, 0, arena_bytes=peak0 + MiB)
    big.load_params(params)
    big.force_plan(0)
    loss0, peak_full, _ = big.train_step(tokens, labels)
    assert loss0 == loss and peak_full == peak0 and peak_full > budget
    G0 = big.grads()
    for k in G0:
        assert np.array_equal(G0[k], G1[k]), k
    big.close()
    # the same batch against the oracle (float32 build, bf16-rounded weights): T = 16384 tokens, a
    # non-empty plan, eight key tiles per head, the full-size tile grids and split reductions
    print("oracle step at B=32, L=512 ...", flush=True)
    ref_loss, RG = oracle_step(shape, params, tokens, labels, np.float32)
    assert abs(loss - ref_loss) <= 1e-2 * abs(ref_loss), (loss, ref_loss)
    worst = check_grads(G1, RG, 2e-2)
    print("bert_base L=512 plan", bin(plan), "loss", loss, ref_loss, "worst grad", worst)


@pytest.mark.parametrize("name,B,L,plan", [
    ("bert_large", 2, 128, 0), ("bert_large", 2, 304, 0x0F0F0F),
    ("gpt2_medium", 2, 129, 0), ("gpt2_medium", 2, 300, 0xAAAAAA),
    ("bert_large_stress", 4, 40, 0), ("bert_large_stress", 2, 384, 0xFFFFFF),
])
def test_other_workload_shapes_reduced_batch(name, B, L, plan):
    """The larger model shapes (BERT-large, GPT-2-medium causal pre-LN) at a reduced batch so the
    oracle finishes in seconds: loss and every gradient against the oracle, with and without
    dropped layers."""
    wl = synthdata.WORKLOADS[name]
    shape = wl.shape
    params = synthdata.make_params(shape, wl.seed)
    tokens, labels = synthdata.make_batch(shape, B, L, 77)
    m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=6144 * MiB)
    m.load_params(params)
    m.force_plan(plan)
    loss, peak, got, worst = check_against_oracle(shape, m, params, tokens, labels, 1e-2, 2e-2, np.float32)
    assert got == plan
    print(name, B, L, "loss", loss, "worst grad", worst)
    m.close()


def test_queued_steps_equal_waited_steps():
    """Iterations issued with loss = NULL (the call returns while the device still works, the pinned
    staging buffers take turns) give the losses, plans, peaks and gradient bits of iterations that
    wait, with the parameter update between them and lengths that change from step to step."""
    shape = SMALL["bf16_postln"]
    params = synthdata.make_params(shape, 31, perturb=True)
    lens = [40, 96, 8, 64, 33, 96, 17]
    batches = [synthdata.make_batch(shape, 4, L, 300 + i) for i, L in enumerate(lens)]
    runs = []
    for wait in (True, False):
        m = mi.Mimose(synthdata.shape_dict(shape), 0, arena_bytes=256 * MiB)
        m.load_params(params)
        m.optimizer_init(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
        m.force_plan(0b101)
        out = []
        for t, l in batches:
            loss, peak, plan = m.train_step(t, l, wait=wait)
            assert (loss is None) == (not wait)
            m.optimizer_step()
            out.append((peak, plan))
        last = m.sync_loss()
        runs.append((out, last, m.grads(), m.params()))
        m.close()
    (o0, l0, g0, p0), (o1, l1, g1, p1) = runs
    assert o0 == o1 and l0 == l1
    for k in g0:
        assert np.array_equal(g0[k], g1[k]), k
        assert np.array_equal(p0[k], p1[k]), k


def test_two_forward_collector_changes_no_bits():
    """Sheltered iterations with every block's forward run twice (the paper's collector to the letter),
    dropout on: losses, gradients, collected samples and the later plans are those of the default
    collector, which runs each forward once."""
    wl = synthdata.WORKLOADS["tiny"]
    shape, B = wl.shape, wl.batch
    d = synthdata.shape_dict(shape)
    cal = mi.Mimose(d, 0, device=None)
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, shape.max_seq)
    cal.close()
    params = synthdata.make_params(shape, wl.seed, perturb=True)
    lens = synthdata.seq_lengths(wl.length_recipe, 14, wl.seed)
    runs = []
    for mode in ("marks", "two_forwards"):
        m = mi.Mimose(d, int(wl.budget_frac * peak0))
        m.set_collector(mode)
        m.set_dropout(0.1, 0.1, 5, 0)
        m.load_params(params)
        out = []
        for i, L in enumerate(lens):
            t, l = synthdata.make_batch(shape, B, L, synthdata.step_seed(wl.seed, i))
            out.append(m.train_step(t, l) + (mi.mimose_get_step_memory(m.ctx, shape.n_layers),))
        runs.append((out, m.grads(), m.stats()["sheltered_steps"]))
        m.close()
    assert runs[0][0] == runs[1][0] and runs[0][2] == runs[1][2] == 10
    for k in runs[0][1]:
        assert np.array_equal(runs[0][1][k], runs[1][1][k]), k


@pytest.mark.parametrize("name,responsive", [("bert_large", 6), ("gpt2_medium", 6), ("bert_large_stress", 6)])
def test_larger_workloads_on_device_under_their_budget(name, responsive):
    """The larger workloads with their own batch size, length recipe and budget fraction on the
    device: the sheltered phase and some responsive iterations.  Every measured peak stays under the
    budget, equals the peak model on the measured components, and every plan is the oracle planner's
    for the same samples; the loss sits at its closed-form initial value."""
    wl = synthdata.WORKLOADS[name]
    shape, B, n = wl.shape, wl.batch, wl.shape.n_layers
    d = synthdata.shape_dict(shape)
    cal = mi.Mimose(d, 0, device=None)
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, shape.max_seq)
    cal.close()
    budget = int(wl.budget_frac * peak0)
    m = mi.Mimose(d, budget)
    m.load_params(synthdata.make_params(shape, wl.seed))
    ref = op.Planner(n, budget, guard=4096)
    lens = synthdata.seq_lengths(wl.length_recipe, 10 + responsive, wl.seed)
    lens[10] = shape.max_seq                       # the longest input among the responsive ones
    expect = np.log(shape.vocab) + 0.5 * 0.02 ** 2 * shape.hidden
    nonempty = 0
    for i, L in enumerate(lens):
        tokens, labels = synthdata.make_batch(shape, B, int(L), synthdata.step_seed(wl.seed, i))
        sheltered = ref.sheltered()
        loss, peak, plan = m.train_step(tokens, labels)
        print(name, "step", i, "L", int(L), "plan", bin(plan), "peak/budget", round(peak / budget, 4), flush=True)
        assert peak <= budget and abs(loss - expect) < 0.03 * expect
        mem = m.step_memory()
        c = op.Components(F=mem["F"], e=mem["e"], g=mem["g"], a=mem["a"], b=mem["b"], w=mem["w"])
        assert peak == op.simulate_peak(c, plan)
        x = B * int(L)
        if sheltered:
            assert plan == (1 << n) - 1
            for l in range(n):
                ref.feed(x, op.Q_A, l, c.a[l]); ref.feed(x, op.Q_B, l, c.b[l]); ref.feed(x, op.Q_W, l, c.w[l])
            ref.feed(x, op.Q_E, -1, c.e); ref.feed(x, op.Q_G, -1, c.g); ref.feed(x, op.Q_F, -1, c.F)
            ref.end_sheltered_step(x)
        else:
            assert plan == ref.query(x).plan
            nonempty += plan != 0
    assert nonempty >= 1 and m.stats()["replans"] == 0
    m.close()
