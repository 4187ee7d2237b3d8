#!/usr/bin/env python3
"""Benchmark of the SAME Gibbs LDA sweep on one MI355X.

A step is one full sweep (zero, draw and scatter over every nonzero, parameter update) of the
news-shaped workload: D=300,000 documents (the last 10% held out), V=100,000 words, K=256
topics, m=100 copies per token, synthetic LDA-generated counts resident in HBM.  Prints one
JSON line: tokens/s per sweep, the HBM-roofline figure of the draw kernel (algorithmic bytes over
its HIP-event duration) and the CPU oracle's rate on a bounded slice of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def draw_kernel_compulsory_bytes(nnz: int, D: int, V: int, K: int) -> float:
    """Bytes of one draw-and-scatter launch if every array were touched once (phi served from cache after
    its first read): word ids and counts, theta and the new document counts, phi, the new word counts
    read and written."""
    return float(nnz) * 8 + float(D) * (4 + 8 * K) + float(V) * K * 12


def draw_kernel_bytes(nnz: int, D: int, K: int) -> float:
    """Algorithmic bytes of one draw-and-scatter launch: per nonzero its word id, its count and the
    K floats of phi_w; per document its column pointer, the K floats of theta_d and the K new counts."""
    return float(nnz) * (8 + 4 * K) + float(D) * (4 + 8 * K)


def measured_traffic(workload: str, form: str = "multinomial"):
    """HBM bytes per draw-kernel launch and where the figure comes from.  It is not measured in this run: it is
    read from the committed summary of the two rocprofv3 counter runs of this same command (None if absent)."""
    tag = "" if form == "multinomial" else f"_{form}"
    rel = os.path.join("profiles", f"draw_kernel{tag}_{workload}_pmc.md")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("hbm_bytes_per_launch"):
                return (float(line.split("=")[1].split()[0]),
                        f"{rel}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, not measured in this run")
    except OSError:
        pass
    return None, None


def cpu_baseline(X_np, K, alpha, beta, m, m0, G, zipf_s, target_s=12.0, poisson=False, sampled=False):
    """Times one sweep of the oracle (as it stands) on a leading slice of documents sized for ~target_s.  The
    sweep starts from a seeded concentrated state (synth.state: document-topic rows and topic-word columns drawn
    from their Dirichlet priors, as after training), the regime of the GPU figures beside it; nothing the GPU
    computed is given to the oracle."""
    import oracle
    import torch
    from paper_1409_5402_amd import synth
    cores = len(os.sched_getaffinity(0))
    docs = min(X_np.D, 512)
    while True:
        sl = X_np.slice_docs(0, docs)
        o = oracle.OracleLDA(sl, K, alpha, beta, seed=1, m0=m0, G=G)
        c = synth.Corpus(sl.D, sl.V, torch.from_numpy(sl.colptr), torch.from_numpy(sl.rowidx), torch.from_numpy(sl.val))
        theta, phi = synth.state(c, K, alpha, beta, seed=123, zipf_s=zipf_s)
        o.theta, o.phi = theta.numpy(), phi.numpy()
        t0 = time.perf_counter()
        o.sweep_poisson(float(m)) if poisson else (o.sweep_sampled(m) if sampled else o.sweep(m))
        dt = max(time.perf_counter() - t0, 1e-4)
        if dt >= 0.5 * target_s or docs >= X_np.D:
            break
        docs = int(min(X_np.D, max(2 * docs, docs * target_s / dt)))
    return {"value": sl.tokens / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"one sweep over the first {docs} documents ({sl.nnz} nonzeros, {int(sl.tokens)} tokens) "
                      f"of the same corpus, K={K}, m={m}, from a seeded concentrated state (synth.state, seed 123); "
                      f"{dt:.2f} s"}


def stream_bench(args):
    """Stream of minibatches (the abstract-collection shape: 100k documents per minibatch, one sweep each, m
    annealed geometrically from 1 to 100): minibatches wait in pinned host memory; the next one is copied,
    its work list built and its initial pass drawn on the library's second stream while the current sweep runs."""
    import torch
    from paper_1409_5402_amd import binding, schedule, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = synth.PRESETS["abstracts_batch"]
    K, alpha, beta, G = p["K"], p["alpha"], p["beta"], args.tokens_per_draw
    pool = []
    for i in range(4):                                   # four distinct minibatches, visited in turn
        gen = dict(p["gen"]); gen["seed"] = 40 + i; gen["D"] = max(1, int(round(gen["D"] * args.scale)))
        c = synth.generate(device=dev, **gen)
        pool.append((c.D, c.colptr.cpu().pin_memory(), c.rowidx.cpu().pin_memory(), c.val.cpu().pin_memory(),
                     c.tokens, c.nnz))
    total = args.warmup + args.steps
    ms = schedule.geometric(1, 100, total)
    b0 = pool[0]
    g = binding.SameLDA(b0[0], p["gen"]["V"], b0[1], b0[2], b0[3], K, alpha, beta, seed=2, m0=ms[0], tokens_per_draw=G)

    def run(first, count, overlapped):
        tokens = 0.0
        for t in range(first, first + count):
            g.sweep(ms[t], float(schedule.rho(t)))
            tokens += pool[t % 4][4]
            nxt = pool[(t + 1) % 4]
            if overlapped:
                g.stage_batch(nxt[0], nxt[1], nxt[2], nxt[3], 1, 0)     # new documents start with one topic per token
                g.commit_batch()
            else:
                g.set_batch(nxt[0], nxt[1], nxt[2], nxt[3], 1)
        g.synchronize()
        return tokens

    run(0, args.warmup, True)
    g.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = run(args.warmup, args.steps, True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    draw_ms, launches = g.get_timing()
    t0 = time.perf_counter()
    tokens_seq = run(args.warmup, args.steps, False)     # the same minibatches and m again, without overlap
    torch.cuda.synchronize()
    dt_seq = time.perf_counter() - t0
    g.get_timing()
    g.close()
    nnz = sum(pool[t % 4][5] for t in range(args.warmup, args.warmup + args.steps))
    docs = sum(pool[t % 4][0] for t in range(args.warmup, args.warmup + args.steps))
    bytes_total = draw_kernel_bytes(nnz, docs, K)
    achieved = bytes_total / (draw_ms * 1e-3) / 1e9
    out = {
        "metric": "streamed tokens/sec, one SAME sweep per minibatch of 100k documents from pinned host memory (K=256, m 1->100)",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"abstracts stream (LDA-generated minibatches, scale {args.scale})", "K": K,
                   "minibatch_docs": pool[0][0], "minibatch_nnz": pool[0][5], "minibatch_tokens": pool[0][4],
                   "m_schedule": f"geometric 1 -> 100 over {total} minibatches", "m_init": 1, "tokens_per_draw": G,
                   "without_overlap_tokens_per_s": tokens_seq / dt_seq,
                   "without_overlap_ms_per_step": 1e3 * dt_seq / args.steps},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "draw_kernel",
                     "kernel_ms": draw_ms / max(launches, 1), "bytes_per_launch": bytes_total / args.steps},
    }
    print(json.dumps(out))


def stats_bench(args):
    """Event counts of the draw kernel (an event-counting build of the library, paper_1409_5402_amd/build.py
    --stats): steps, trips, pmf terms and shared passes per task at three states of the news-shaped workload -
    the first sweep at m after the random start (flat posteriors), the last burn-in sweep at m=1, and the
    converged state the headline is timed at."""
    import ctypes
    import torch
    from paper_1409_5402_amd import binding, build, synth

    newest = max(os.path.getmtime(os.path.join(dp, f)) for dp, _, fs in os.walk(os.path.join(ROOT, "paper_1409_5402_amd", "csrc"))
                 for f in fs)
    if not os.path.exists(build.STATS_LIB) or os.path.getmtime(build.STATS_LIB) < newest:
        build.build(stats=True)
    L = binding.load(build.STATS_LIB)
    L.same_lda_stats_buffer.argtypes = [ctypes.c_void_p]
    L.same_lda_stats_buffer.restype = None
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = synth.PRESETS[args.workload]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], args.tokens_per_draw
    corpus = synth.preset(args.workload, device=dev, scale=args.scale)
    n_train = corpus.D - corpus.D // 10 if corpus.D >= 10 else corpus.D
    train = corpus.slice_docs(0, n_train)
    stats = torch.zeros(48, dtype=torch.int64, device=dev)

    def measured(g, mm, what):
        stats.zero_()
        L.same_lda_stats_buffer(stats.data_ptr())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.sweep(mm)
        g.synchronize()
        ms = 1e3 * (time.perf_counter() - t0)
        L.same_lda_stats_buffer(None)
        v = stats.cpu().numpy()
        nt = g.task_count
        nw = (nt + 63) // 64
        return {"state": what, "m": mm, "sweep_ms_with_counters": round(ms, 2),
                "steps_per_task": round(v[1] / nt, 3), "trips_per_64_tasks": round(v[2] / nw, 2),
                "block_reloads_per_task": round(v[3] / nt, 3),
                "pmf_terms_per_task": round(v[4] / nt, 3), "binomials_per_task": round(v[5] / nt, 3),
                "shared_passes_per_64_tasks": round(v[6] / nw, 4), "shared_pieces_per_64_tasks": round(v[7] / nw, 3),
                "lanes_per_trip": {"stepping": round(v[8] / max(v[2], 1), 2), "walking_on": round(v[9] / max(v[2], 1), 2),
                                   "waiting_for_a_shared_pass": round(v[10] / max(v[2], 1), 2),
                                   "idle": round(v[11] / max(v[2], 1), 2)},
                "pmf_rounds_per_trip": round(v[12] / max(v[2], 1), 3), "refills_per_64_tasks": round(v[13] / nw, 3),
                "chunks_per_task": round(v[15] / nt, 4), "chunk_batches_per_64_tasks": round(v[14] / nw, 4),
                "counts_sent_straight_to_a_word_row_with_a_full_slot_per_task": round(sum(v[16:22]) / nt, 4),
                "of_them_by_group_size_1_2_4_8_16_32up": [int(x) for x in v[16:22]],
                "of_them_by_word_id_below_16_256_4096_rest": [int(x) for x in v[22:26]]}

    out = []
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta, seed=2, m0=1,
                        tokens_per_draw=G)
    out.append(measured(g, m, f"first sweep at m={m} after the random start"))
    g.close()
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta, seed=2, m0=1,
                        tokens_per_draw=G)
    for _ in range(args.burn_in[0] - 1):
        g.sweep(1)
    out.append(measured(g, 1, f"sweep {args.burn_in[0]} of the burn-in at m=1"))
    for _ in range(args.burn_in[1] + args.warmup):
        g.sweep(m)
    out.append(measured(g, m, f"converged state: {args.burn_in[0]} sweeps at m=1, {args.burn_in[1] + args.warmup} at m={m}"))
    theta_s, phi_s = synth.state(train, K, alpha, beta, seed=123, zipf_s=p["gen"].get("zipf_s", 0.0))
    g.set(binding.THETA, theta_s)
    g.set(binding.PHI, phi_s)
    out.append(measured(g, m, "seeded concentrated state (synth.state, seed 123)"))
    g.close()
    print(json.dumps({"workload": f"{args.workload} (scale {args.scale})", "K": K, "tokens_per_draw": G, "states": out}))


def sddmm_bench(args):
    """The normaliser of Algorithm 3 alone (SDDMM, Section 5.3) over the news-shaped matrix at full size."""
    import torch
    from paper_1409_5402_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = synth.PRESETS[args.workload]
    K = p["K"]
    corpus = synth.preset(args.workload, device=dev, scale=args.scale)
    n_train = corpus.D - corpus.D // 10 if corpus.D >= 10 else corpus.D
    train = corpus.slice_docs(0, n_train)
    st = train.stats()
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, p["alpha"], p["beta"],
                        seed=2, m0=1, tokens_per_draw=args.tokens_per_draw)
    for _ in range(5):
        g.sweep(1)                                       # a non-trivial theta / phi
    mu = torch.empty(train.nnz, dtype=torch.float32, device=dev)
    warm = min(args.warmup, 10)
    for _ in range(warm):
        g.sddmm(mu)
    g.synchronize()
    g.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.sddmm(mu)
    g.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, launches = g.get_timing()
    g.close()
    bytes_per_launch = float(st["nnz"]) * (12 + 4 * K) + float(st["D"]) * 4 * K   # ids, phi row, mu; theta rows once
    achieved = bytes_per_launch / (kernel_ms / launches * 1e-3) / 1e9
    print(json.dumps({
        "metric": "nonzeros/sec of the stand-alone SDDMM normaliser (K=256) + achieved HBM GB/s vs 8 TB/s",
        "value": st["nnz"] / (dt / args.steps), "unit": "nonzeros/s", "n_gpus": 1, "steps": args.steps, "warmup": warm,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} (LDA-generated, scale {args.scale})", "D": st["D"], "V": st["V"], "K": K,
                   "nnz": st["nnz"]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "sddmm_small_kernel" if (K % 4 == 0 and K <= 256) else "sddmm_kernel",
                     "kernel_ms": kernel_ms / launches, "bytes_per_launch": bytes_per_launch}}))


def vb_bench(args):
    """The E-step of online variational Bayes LDA (the second consumer of the normaliser, Section 5.3) over the
    news-shaped matrix at full size: `--vb-iters` iterations per document from gamma = 1, lambda a seeded
    concentrated topic-word state."""
    import torch
    from paper_1409_5402_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = synth.PRESETS[args.workload]
    K = p["K"]
    corpus = synth.preset(args.workload, device=dev, scale=args.scale)
    n_train = corpus.D - corpus.D // 10 if corpus.D >= 10 else corpus.D
    train = corpus.slice_docs(0, n_train)
    st = train.stats()
    _, phi_s = synth.state(train, K, p["alpha"], p["beta"], seed=123, zipf_s=p["gen"].get("zipf_s", 0.0))
    lam = (0.01 + phi_s * (float(st["tokens"]) / K)).contiguous()
    del phi_s
    g = binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, p["alpha"], p["beta"],
                        seed=2, m0=1, tokens_per_draw=args.tokens_per_draw)
    b = torch.empty_like(lam)
    shift = torch.empty(train.V, dtype=torch.float32, device=dev)
    gamma = torch.empty((train.D, K), dtype=torch.float32, device=dev)
    log_mu = torch.empty(train.nnz, dtype=torch.float32, device=dev)
    alpha, iters = 0.1, args.vb_iters

    def step():
        gamma.fill_(1.0)
        g.vb_exp_elog_beta(lam, b, shift)
        g.vb_estep(b, shift, alpha, iters, gamma, log_mu)

    warm = min(args.warmup, 3)
    for _ in range(warm):
        step()
    g.synchronize()
    g.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    g.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, launches = g.get_timing()
    bound = float((log_mu.double() * train.val.double()).sum() / st["tokens"])      # sum c log mu / tokens
    g.close()
    # per iteration: word id, count and the b row of every nonzero; per launch: gamma read and written, log mu written
    bytes_per_launch = float(iters) * float(st["nnz"]) * (8 + 4 * K) + float(st["D"]) * 8 * K + 4.0 * float(st["nnz"])
    achieved = bytes_per_launch / (kernel_ms / launches * 1e-3) / 1e9
    print(json.dumps({
        "metric": f"tokens/sec of the variational E-step ({iters} iterations per document, K={K}) + achieved HBM GB/s vs 8 TB/s",
        "value": st["tokens"] / (dt / args.steps), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": warm,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} (LDA-generated, scale {args.scale})", "D": st["D"], "V": st["V"], "K": K,
                   "nnz": st["nnz"], "tokens": st["tokens"], "vb_iters": iters, "alpha": alpha,
                   "step": "exp E[log beta] of lambda, then the E-step of all documents from gamma = 1",
                   "mean_log_mu_per_token": bound},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "vb_estep_kernel",
                     "kernel_ms": kernel_ms / launches, "bytes_per_launch": bytes_per_launch}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps right before the timed ones, same kind as the timed ones "
                         "(default 10; 20 minibatches in stream mode)")
    ap.add_argument("--burn-in", type=int, nargs=2, default=[100, 30], metavar=("AT_M1", "AT_M"),
                    help="resident mode: state preparation before the warm-up, untimed: sweeps at m=1 (an annealing "
                         "burn-in that breaks the symmetry of the random start), then sweeps at the workload's m.  "
                         "With the defaults the timed sweeps complete a 50-sweep run at m from a converged state")
    ap.add_argument("--workload", default="news")
    ap.add_argument("--scale", type=float, default=1.0, help="fraction of the workload's documents (1.0 = full size)")
    ap.add_argument("--tokens-per-draw", type=int, default=None, help="default: binding.DEFAULT_TOKENS_PER_DRAW")
    ap.add_argument("--form", choices=["multinomial", "poisson"], default="multinomial",
                    help="form of the factored draw: the exact-total multinomial (the headline path) or the "
                         "independent Poisson counts of Algorithm 3 as printed")
    ap.add_argument("--update", choices=["collapsed", "sampled"], default="collapsed",
                    help="parameter step: the posterior means of Eq. 6 (what the paper runs, the headline) or "
                         "Dirichlet draws of theta and phi (Algorithm 2, third step; multinomial form only)")
    ap.add_argument("--mode", choices=["resident", "stream", "sddmm", "stats", "vb"], default="resident",
                    help="resident: sweeps over one matrix held in HBM (the headline); stream: one sweep per "
                         "minibatch of a stream of host-resident minibatches; sddmm: the normaliser alone; "
                         "stats: event counts of the draw kernel from a counting build of the library; "
                         "vb: the E-step of online variational Bayes LDA on the same matrix")
    ap.add_argument("--vb-iters", type=int, default=5, help="vb mode: iterations per document")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-spec-run", action="store_true",
                    help="skip the legs beside the headline: the workload's specified run from the random start "
                         "(first_sweep_ms, runN_mean_ms) and the sweep from the seeded synthetic state")
    ap.add_argument("--no-loglik", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.tokens_per_draw is None:
        from paper_1409_5402_amd.binding import DEFAULT_TOKENS_PER_DRAW
        args.tokens_per_draw = DEFAULT_TOKENS_PER_DRAW
    if args.mode == "stream":
        if args.warmup is None:
            args.warmup, args.steps = 20, max(args.steps, 40)
        return stream_bench(args)
    if args.warmup is None:
        args.warmup = 10
    if args.mode == "sddmm":
        return sddmm_bench(args)
    if args.mode == "vb":
        return vb_bench(args)
    if args.mode == "stats":
        return stats_bench(args)
    import oracle
    from paper_1409_5402_amd import binding, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = synth.PRESETS[args.workload]
    K, m, alpha, beta, G = p["K"], p["m"], p["alpha"], p["beta"], args.tokens_per_draw

    t0 = time.perf_counter()
    corpus = synth.preset(args.workload, device=dev, scale=args.scale)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t0
    n_train = corpus.D - corpus.D // 10 if corpus.D >= 10 else corpus.D
    train = corpus.slice_docs(0, n_train)
    test = corpus.slice_docs(n_train, corpus.D) if n_train < corpus.D else None
    st = train.stats()

    m0 = 1      # random initialisation: one topic per token
    poisson = args.form == "poisson"
    sampled = args.update == "sampled"
    if poisson and sampled:
        sys.exit("bench.py: --update sampled goes with the multinomial form")

    def make():
        return binding.SameLDA(train.D, train.V, train.colptr, train.rowidx, train.val, K, alpha, beta,
                               seed=2, m0=m0, tokens_per_draw=G)

    def sweeper(h):
        return ((lambda mm: h.sweep_poisson(float(mm))) if poisson else
                (lambda mm: h.sweep_sampled(mm)) if sampled else (lambda mm: h.sweep(mm)))

    # The run the workload specifies, from the library's own random start and without any burn-in: p["sweeps"]
    # sweeps at m; every sweep is timed on its own (wall clock around a synchronised call).
    spec = {}
    if not args.no_spec_run:
        g = make()
        sw = sweeper(g)
        per = []
        for _ in range(p["sweeps"]):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sw(m)
            g.synchronize()
            per.append(1e3 * (time.perf_counter() - t0))
        spec = {"first_sweep_ms": per[0], f"run{len(per)}_mean_ms": sum(per) / len(per), f"run{len(per)}_last_ms": per[-1],
                "spec_run": f"{len(per)} sweeps at m={m} right after same_lda_init (one random topic per token), no burn-in"}
        # one sweep from the seeded concentrated state the oracle's cpu_baseline leg is timed on
        theta_s, phi_s = synth.state(train, K, alpha, beta, seed=123, zipf_s=p["gen"].get("zipf_s", 0.0))
        g.set(binding.THETA, theta_s)
        g.set(binding.PHI, phi_s)
        del theta_s, phi_s
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sw(m)
        g.synchronize()
        spec["synth_state_sweep_ms"] = 1e3 * (time.perf_counter() - t0)
        g.close()

    t0 = time.perf_counter()
    g = make()
    t_init = time.perf_counter() - t0
    sweep = sweeper(g)
    for _ in range(args.burn_in[0]):        # state preparation: the sampler is timed where a run spends its time,
        sweep(1)                            # with topics formed, not in the first sweeps after a random start
    for _ in range(args.burn_in[1]):
        sweep(m)
    for _ in range(args.warmup):
        sweep(m)
    g.synchronize()
    g.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sweep(m)
    g.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    draw_ms, launches = g.get_timing()
    g.set_timing(False)
    assert launches == args.steps

    ms_per_step = 1e3 * dt / args.steps
    tokens_per_s = st["tokens"] / (dt / args.steps)
    bytes_per_launch = draw_kernel_bytes(st["nnz"], st["D"], K)
    draw_ms_avg = draw_ms / launches
    achieved = bytes_per_launch / (draw_ms_avg * 1e-3) / 1e9

    traffic, traffic_source = measured_traffic(args.workload, args.form)
    out = {
        "metric": ("tokens/sec per SAME sweep in the Poisson form (K=256, m=100) + achieved HBM GB/s vs 8 TB/s" if poisson else
                   "tokens/sec per SAME sweep with sampled theta and phi (K=256, m=100) + achieved HBM GB/s vs 8 TB/s" if sampled else
                   "tokens/sec per SAME sweep (K=256, m=100) + achieved HBM GB/s vs 8 TB/s"),
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} (LDA-generated, scale {args.scale})", "D": st["D"], "V": st["V"],
                   "K": K, "m": m, "nnz": st["nnz"], "tokens": st["tokens"], "max_count": st["max_count"],
                   "form": args.form, "update": args.update, "tokens_per_draw": G, "draw_tasks": g.task_count, "alpha": alpha, "beta": beta,
                   "m_init": m0,
                   "state": f"untimed before the warm-up: {args.burn_in[0]} sweeps at m=1 then {args.burn_in[1]} at m={m}",
                   **spec, "generate_s": round(t_gen, 2), "init_s": round(t_init, 2)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "draw_kernel", "kernel_ms": draw_ms_avg, "bytes_per_launch": bytes_per_launch,
                     "compulsory_bytes_per_launch": draw_kernel_compulsory_bytes(st["nnz"], st["D"], st["V"], K)},
    }
    if test is not None and not args.no_loglik:
        out["config"]["heldout_ll_per_word"] = g.loglik(test.D, test.colptr, test.rowidx, test.val, 3, m)
    g.close()

    if not args.no_cpu_baseline:
        X_np = oracle.CSC(train.D, train.V, train.colptr.cpu().numpy(), train.rowidx.cpu().numpy(),
                          train.val.cpu().numpy())
        out["cpu_baseline"] = cpu_baseline(X_np, K, alpha, beta, m, m0, G, p["gen"].get("zipf_s", 0.0),
                                           poisson=poisson, sampled=sampled)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
