"""Throughput of the checkpointed variable-length training step on one MI355X.

One step = one call of mimose_train_step: plan lookup, embedding, all layers forward with the
plan's drops, head + loss, backward with recomputation, embedding backward.  Prints one JSON
line: samples/s, the bf16 MFMA roofline of the GEMM kernel measured with events on the work
stream, and the CPU oracle timed on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
GEMM_SOURCES = ("gemm.hip", "gemm_dma.hip", "gemm_pp.hip", "gemm_device.h")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bert_base_gemm_hbm_traffic.txt")


def recorded_gemm_traffic(workload):
    """HBM bytes per GEMM launch from the committed FETCH_SIZE / WRITE_SIZE summary, or None when
    the GEMM sources have changed since the counters were taken (or another workload runs)."""
    import hashlib
    if workload != "bert_base" or not os.path.exists(TRAFFIC_FILE):
        return None
    kv = {}
    for line in open(TRAFFIC_FILE):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    sha = hashlib.sha256()
    for f in GEMM_SOURCES:
        sha.update(open(os.path.join(ROOT, "paper_2209_02478_amd", "csrc", f), "rb").read())
    if kv.get("sources_sha256") != sha.hexdigest():
        return None
    return int(kv["traffic_bytes_per_launch"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="bert_base")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plan-mode", default="input_aware", choices=["input_aware", "static_max", "all", "none"],
                    help="planning policy of the responsive phase (default: the paper's input-aware planner; "
                         "static_max = one plan for the longest sequence, as a static planner would make; "
                         "none ignores the budget)")
    ap.add_argument("--no-update", action="store_true",
                    help="leave the parameter update (AdamW) out of the iteration: forward, loss and backward only")
    ap.add_argument("--cost-aware", action="store_true",
                    help="use the forward times collected in the sheltered steps inside Algorithm 1's buckets")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout probability of the attention probabilities and of the hidden sites (embedding output, attention and feed-forward "
                         "block outputs), masks from the counter-based generator; 0 = off, the measured default")
    ap.add_argument("--size-quantum", type=int, default=1,
                    help="plan-cache key granularity in tokens (Section 5: similar input sizes share a plan): a batch of x tokens "
                         "uses the plan made for x rounded up to a multiple of this; 1 = exact sizes")
    ap.add_argument("--collector", default="marks", choices=["marks", "two_forwards"],
                    help="how the sheltered iterations measure a block: from the allocator's marks in one forward (default), "
                         "or with the paper's two forwards per block (Section 4.2), whose cost the overhead object then shows")
    ap.add_argument("--hbm-kernels", action="store_true",
                    help="instead of the training run: launch every HBM-bound kernel of the step on its own, through the "
                         "kernel-level entry points, at the BERT-base median size and at the BERT-large stress size, and "
                         "print their algorithmic bytes, durations and GB/s (run it under rocprofv3 --kernel-trace for the "
                         "kernels' own durations)")
    ap.add_argument("--wait-every-step", action="store_true",
                    help="read the loss after every iteration (the host blocks until the device is done) instead of "
                         "queueing the timed iterations one after the other and reading the loss once at the end")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 256 MiB element-wise copy kernels (reference for scaling FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
                         "(no collectives or sharding exist in this library)\n")
        sys.exit(2)

    import numpy as np
    import torch
    import synthdata
    import paper_2209_02478_amd as mi

    if not os.path.exists(mi.LIB_PATH):
        from paper_2209_02478_amd import build as b
        b.build(verbose=False)
    if args.hbm_kernels:
        print(json.dumps(hbm_kernels(mi, torch)))
        return
    wl = synthdata.WORKLOADS[args.workload]
    shape, B, N = wl.shape, wl.batch, wl.shape.n_layers
    d = synthdata.shape_dict(shape)

    update = not args.no_update
    adamw = dict(lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    cal = mi.Mimose(d, 0, device=None)
    if update:
        cal.optimizer_init(**adamw)           # its state is part of the fixed memory the budget is a fraction of
    cal.force_plan(0)
    peak0, _ = cal.dry_step(B, shape.max_seq)
    cal.close()
    budget = int(wl.budget_frac * peak0)

    if args.plan_mode == "none":                      # the no-checkpoint limit needs the whole peak
        m = mi.Mimose(d, 0, arena_bytes=peak0 + (1 << 20))
    else:
        m = mi.Mimose(d, budget, cost_aware=int(args.cost_aware), size_quantum=args.size_quantum)
    m.set_plan_mode(args.plan_mode)
    m.set_collector(args.collector)
    m.load_params(synthdata.make_params(shape, wl.seed))
    if update:
        m.optimizer_init(**adamw)
    if args.dropout > 0:
        m.set_dropout(args.dropout, args.dropout, wl.seed, 0)

    def iteration(t, l, wait=True):
        r = m.train_step(t, l, wait=wait)
        if update:
            m.optimizer_step()
        return r

    sheltered = 10
    total = sheltered + args.warmup + args.steps
    lens = synthdata.seq_lengths(wl.length_recipe, total, wl.seed)
    last_note = [time.perf_counter()]

    def note(what):                           # a line on stderr every half minute of a long run
        if time.perf_counter() - last_note[0] > 30:
            sys.stderr.write(f"bench.py: {what}\n")
            sys.stderr.flush()
            last_note[0] = time.perf_counter()

    batches = []
    for i, L in enumerate(lens):
        batches.append(synthdata.make_batch(shape, B, L, synthdata.step_seed(wl.seed, i)))
        note(f"made batch {i + 1} of {total}")

    if args.pmc_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)        # an elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    t_sheltered = []                          # the collecting iterations, one by one
    for i, (t, l) in enumerate(batches[:sheltered + args.warmup]):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        iteration(t, l)
        torch.cuda.synchronize()
        if i < sheltered:
            t_sheltered.append(time.perf_counter() - t0)
    timed = batches[sheltered + args.warmup:]
    s0 = m.stats()
    max_peak = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i, (t, l) in enumerate(timed):        # queued one after the other; the loss is read once, at the end
        _, pk, _ = iteration(t, l, wait=args.wait_every_step)
        max_peak = max(max_peak, pk)
        note(f"timed iteration {i + 1} of {len(timed)} issued")
    last_loss = m.sync_loss()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert np.isfinite(last_loss)
    s1 = m.stats()

    # Overhead accounting in the manner of Section 6.4: what a collecting iteration costs beyond the
    # same batch under its responsive plan, and what generating the plans cost
    t_again = []
    if args.plan_mode == "input_aware":
        for t, l in batches[:sheltered]:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            iteration(t, l)
            torch.cuda.synchronize()
            t_again.append(time.perf_counter() - t0)
    s2 = m.stats()

    # same steps again with per-kernel events on the work stream
    mi.mimose_profile_enable(m.ctx, 1)
    for i, (t, l) in enumerate(timed):
        iteration(t, l)
        note(f"per-kernel timing pass, iteration {i + 1} of {len(timed)}")
    torch.cuda.synchronize()
    upd = None
    if update:                                # the update alone, back to back, on the context's stream
        n_elems = sum(int(np.prod(sh)) for sh in m.shapes.values())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            m.optimizer_step()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 100.0
        per_elem = 28 + (2 if shape.dtype == "bf16" else 0)     # read g, m, v, p; write m, v, p (+ bf16 copy)
        upd = {"kind": "adamw, one launch over all tensors, inside the timed iteration", "avg_us": round(us, 1),
               "gbs": round(n_elems * per_elem / (us * 1e-6) / 1e9, 1)}
    kernels = {}
    gemm_flops_per_launch = 0.0
    for i, name in enumerate(mi.KERNEL_CLASSES):
        n, ms, work = mi.mimose_profile_read(m.ctx, i)
        if n and i == 0:
            gemm_flops_per_launch = work / n
        if n:
            rate = work / (ms * 1e-3)
            kernels[name] = {"launches": n, "avg_us": round(1e3 * ms / n, 3),
                             ("tflops" if i < 3 else "gbs"): round(rate / (1e12 if i < 3 else 1e9), 2)}
    mi.mimose_profile_enable(m.ctx, 0)
    m.close()

    K = len(timed)
    useful = s1["useful_flops_total"] - s0["useful_flops_total"]
    recompute = s1["recompute_flops_total"] - s0["recompute_flops_total"]
    hits = s1["cache_hits"] - s0["cache_hits"]
    misses = s1["cache_misses"] - s0["cache_misses"]
    gemm_tflops = kernels.get("gemm", {}).get("tflops", 0.0)
    out = {
        "metric": "train samples/s under fixed mem budget, BERT-base var seq len",
        "value": round(K * B / dt, 2), "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(1e3 * dt / K, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {N} layers, hidden {shape.hidden}, {shape.n_heads} heads, ffn "
                               f"{'/'.join(map(str, shape.ffn_by_layer)) if shape.ffn_by_layer else shape.ffn}, "
                               f"vocab {shape.vocab}, batch {B}, per-batch length {wl.length_recipe}, "
                               f"budget {wl.budget_frac:.2f} x no-checkpoint peak at L={shape.max_seq}",
                   "global_batch": B, "mean_seq_len": round(float(np.mean([t.shape[1] for t, _ in timed])), 1),
                   "budget_bytes": budget, "sheltered_steps": sheltered, "plan_mode": args.plan_mode, "collector": args.collector, "size_quantum": args.size_quantum,
                   "cost_aware": bool(args.cost_aware), "dropout": args.dropout,
                   "iteration": "forward + loss + backward + AdamW update (fp32 moments and master weights)" if update
                                else "forward + loss + backward (no parameter update)",
                   "host_waits_every_step": bool(args.wait_every_step)},
        "tokens_per_s": round(sum(t.size for t, _ in timed) / dt, 1),
        "useful_tflops": round(useful / dt / 1e12, 2), "recompute_tflops": round(recompute / dt / 1e12, 2),
        "mfma_frac_useful": round(useful / dt / 1e12 / PEAK_BF16_TFLOPS, 4),
        "mfma_frac_useful_plus_recompute": round((useful + recompute) / dt / 1e12 / PEAK_BF16_TFLOPS, 4),
        "recompute_overhead": round(recompute / useful, 4),
        "mean_recomputed_layers": round((s1["recomputed_layers_total"] - s0["recomputed_layers_total"]) / K, 2),
        "plan_cache_hit_rate": round(hits / max(hits + misses, 1), 4),
        "planner_us_per_step": round((s1["planner_ns_total"] - s0["planner_ns_total"]) / K / 1e3, 2),
        "max_peak_over_budget": round(max_peak / budget, 4),
        "kernels": kernels,
        "kernels_timing": "gemm: events bound to each kernel's own start and end; other classes: markers around the launch, "
                          "which read a few microseconds more than the kernel itself (see profiles/ for the kernel trace)",
        "update": upd,
        "roofline": {"bound": "mfma", "kernel": "bgemm_kernel / bgemm_dma_kernel / bgemm_pp_kernel (every product of the timed steps, the reduction kernel of a split product included)",
                     "achieved": gemm_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / PEAK_BF16_TFLOPS, 4),
                     "avg_launch_us": kernels.get("gemm", {}).get("avg_us"),
                     "flops_per_launch": round(gemm_flops_per_launch),
                     "traffic": recorded_gemm_traffic(args.workload)},
    }
    if t_again:
        extra = [1e3 * (a - b) for a, b in zip(t_sheltered, t_again)]
        gen_ms = s2["plan_gen_ns_total"] / 1e6
        total = sum(extra) + gen_ms
        out["overhead"] = {
            "collector_ms_per_sheltered_iteration": {"first": round(extra[0], 3), "median": round(float(np.median(extra)), 3),
                                                     "mean": round(float(np.mean(extra)), 3)},
            "sheltered_iterations": sheltered,
            "plan_generation_us": {"min": round(s2["plan_gen_ns_min"] / 1e3, 2), "max": round(s2["plan_gen_ns_max"] / 1e3, 2),
                                   "times": s2["plan_gen_count"]},
            "total_ms": round(total, 3), "total_in_iterations": round(total / (1e3 * dt / K), 3),
            "note": "collector = a sheltered iteration (every layer checkpointed and timed) minus the same batch "
                    "re-run under its responsive plan; the first one also pays the one-time kernel loading"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, update, adamw)
    print(json.dumps(out))


def hbm_kernels(mi, torch):
    """Every HBM-bound kernel alone, bf16, at (T, H, F, V) of the BERT-base median batch (B=32, L=200) and of
    the BERT-large stress batch (B=256, L=512).  Each launch works on buffers of its own, enough of them to
    exceed the 256 MB last-level cache, so the bytes come from HBM.  Algorithmic bytes per token: LayerNorm
    forward 4H (6H from an fp32 sum), backward 6H bf16 (10H with fp32 gradient and input), GELU backward 6F,
    softmax cross-entropy 4V (in place), embedding forward 6H + 4."""
    dev = "cuda:0"
    bf, f32 = torch.bfloat16, torch.float32
    rows = []

    def timed(name, size, bytes_per_launch, n_sets, launch):
        for k in range(min(n_sets, 3)):
            launch(k)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(n_sets, 10)
        e0.record()
        for k in range(reps):
            launch(k % n_sets)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        rows.append({"kernel": name, "size": size, "bytes_per_launch": int(bytes_per_launch), "launches": reps,
                     "avg_us_events": round(us, 2), "gbs": round(bytes_per_launch / (us * 1e-6) / 1e9, 1),
                     "frac_of_8TBs": round(bytes_per_launch / (us * 1e-6) / 8e12, 3)})

    for tag, T, H, F, V in (("bert_base median: T=6400 H=768 F=3072 V=30522", 6400, 768, 3072, 30522),
                            ("bert_large stress: T=131072 H=1024 F=4096 V=30522", 131072, 1024, 4096, 30522)):
        def sets(bytes_one):                      # buffers sets so that the rotation exceeds 512 MB, at most 64
            return int(max(2, min(64, (512 << 20) // max(bytes_one, 1) + 1)))
        gam = torch.ones(H, dtype=bf, device=dev); bet = torch.zeros(H, dtype=bf, device=dev)
        # LayerNorm forward, bf16 rows and fp32 rows (the unrounded residual sum of post-LN blocks)
        n = sets(T * H * 4)
        xs = [torch.randn(T, H, device=dev).to(bf) for _ in range(n)]
        ys = [torch.empty(T, H, dtype=bf, device=dev) for _ in range(n)]
        timed("layernorm_fwd bf16", tag, 4 * H * T, n, lambda k: mi.mimose_op_layernorm_fwd(1, xs[k], 0, gam, bet, ys[k], T, H, 1e-5))
        n = sets(T * H * 6)
        xw = [torch.randn(T, H, device=dev) for _ in range(n)]
        timed("layernorm_fwd fp32 rows in", tag, 6 * H * T, n, lambda k: mi.mimose_op_layernorm_fwd(1, xw[k], 1, gam, bet, ys[k % len(ys)], T, H, 1e-5))
        # LayerNorm backward: fp32 gradient and input (post-LN blocks) and all-bf16
        part = torch.empty(mi.mimose_op_partial_rows(T) * 2 * H, dtype=f32, device=dev)
        dg = torch.empty(H, dtype=f32, device=dev); db = torch.empty(H, dtype=f32, device=dev)
        n = sets(T * H * 10)
        dyw = [torch.randn(T, H, device=dev) for _ in range(n)]
        dxs = [torch.empty(T, H, dtype=bf, device=dev) for _ in range(n)]
        timed("layernorm_bwd fp32 dy and x in", tag, 10 * H * T, n,
              lambda k: mi.mimose_op_layernorm_bwd(1, dyw[k], 1, xw[k % len(xw)], 1, gam, dxs[k], None, dg, db, part, T, H, 1e-5))
        timed("layernorm_bwd bf16", tag, 6 * H * T, len(xs),
              lambda k: mi.mimose_op_layernorm_bwd(1, xs[k], 0, ys[k], 0, gam, dxs[k % len(dxs)], None, dg, db, part, T, H, 1e-5))
        del xw, dyw, dxs, xs, ys
        # GELU backward in place
        n = sets(T * F * 4)
        ds = [torch.randn(T, F, device=dev).to(bf) for _ in range(n)]
        ps = [torch.randn(T, F, device=dev).to(bf) for _ in range(n)]
        timed("gelu_bwd", tag, 6 * F * T, n, lambda k: mi.mimose_op_gelu_bwd(1, ds[k], ps[k], T * F, 0))
        del ds, ps
        # softmax cross-entropy in place (the stress size in chunks of 16384 rows: the logits of 131072 tokens are 8 GB)
        Tx = min(T, 16384)
        ldv = (V + 63) // 64 * 64
        n = sets(Tx * ldv * 2)
        lg = [torch.randn(Tx, ldv, device=dev).to(bf) for _ in range(n)]
        lab = torch.randint(0, V, (Tx,), dtype=torch.int32, device=dev)
        rl = torch.empty(Tx, dtype=f32, device=dev); ls = torch.empty(1, dtype=f32, device=dev)
        timed("softmax_xent", tag if Tx == T else tag + " (rows 16384 at a time)", 4 * ldv * Tx, n,
              lambda k: mi.mimose_op_softmax_xent(1, lg[k], ldv, lab, rl, ls, Tx, V, Tx))
        del lg
        # embedding forward with LayerNorm
        L = 200 if T == 6400 else 512
        B = T // L
        tok = torch.randn(V, H, device=dev).to(bf); pos = torch.randn(512, H, device=dev).to(bf)
        ids = torch.randint(0, V, (T,), dtype=torch.int32, device=dev)
        n = sets(T * H * 4)
        so = [torch.empty(T, H, dtype=bf, device=dev) for _ in range(n)]
        yo = [torch.empty(T, H, dtype=bf, device=dev) for _ in range(n)]
        timed("embed_fwd", tag, (6 * H + 4) * T, n, lambda k: mi.mimose_op_embed_fwd(1, ids, tok, pos, gam, bet, so[k], yo[k], B, L, H, 1e-5, 1))
        del so, yo
    return {"what": "HBM-bound kernels alone, bf16, buffers rotated past the last-level cache; durations from events around "
                    "the launches (a kernel trace of the same command gives the kernels' own)", "peak_gbs": 8000, "kernels": rows}


def cpu_baseline(wl, update, adamw):
    """The oracle as it stands, timed on this host: one step on a reduced batch."""
    import numpy as np
    import synthdata
    from oracle import model as om
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    shape = wl.shape
    L = min(200, shape.max_seq)
    cfg = om.Cfg.from_shape(synthdata.shape_dict(shape))
    # bounded sample: about 4 TFLOP of the same model (a full BERT-base batch at L=200), never
    # more than the workload's batch
    per_sample = om.flops_per_step(cfg, 1, L)[0]
    Bs = int(max(1, min(wl.batch, round(4.3e12 / per_sample))))
    params = synthdata.make_params(shape, wl.seed)
    tokens, labels = synthdata.make_batch(shape, Bs, L, 1)
    t0 = time.perf_counter()
    _, grads = om.train_step(cfg, params, tokens, labels)
    if update:
        from oracle.optimizer import AdamW
        AdamW(**adamw).step(params, grads)
    dt = time.perf_counter() - t0
    what = "forward, loss, backward, update" if update else "forward, loss, backward"
    cpu_model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        nproc = len(os.sched_getaffinity(0))
    except AttributeError:
        nproc = os.cpu_count() or 1
    return {"value": round(Bs / dt, 3), "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "dtype": "f64", "blas_threads": int(cores), "nproc": int(nproc), "cpu_model": cpu_model,
            "sample": f"one fp64 oracle iteration ({what}) of the same model at batch {Bs}, L={L}: {dt:.1f} s"}


if __name__ == "__main__":
    main()
