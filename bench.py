"""Benchmark: matmul-sumcheck prove time per layer and achieved HBM bandwidth on one MI355X.

One step = one full proof of C = A.B for the FFN up-projection shape (A 2048x4096 int16,
B 4096x14336 int8): field encoding of both operands, eq vectors, both streaming partial
evaluations, the 12 sumcheck rounds with their transcript hashing, proof assembly.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure


def recorded_traffic():
    """HBM bytes per launch of the dominant kernel as measured with hardware counters (see
    profiles/reduce_B_ffn_up_hbm_counters.txt); None once the kernel sources have changed since."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "reduce_B_ffn_up_hbm_counters.txt")
    try:
        kv = dict(line.split(" = ", 1) for line in open(path).read().splitlines() if " = " in line and not line.startswith(" "))
        h = hashlib.sha256()
        for fn in ("kernels.hip", "goldilocks_device.h", "kernels.h", "prover.cpp"):   # kernels and launch geometry
            h.update(open(os.path.join(ROOT, "paper_2602_22700_amd", "csrc", fn), "rb").read())
        if h.hexdigest() != kv["kernel_sources_sha256"].strip():
            return None
        return int(kv["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def make_workload(name, torch, imm, workloads):
    """Returns a list of (A_np, B_np, A_dev, B_dev, Commit): the statements of one step."""
    import numpy as np
    if name == "ffn_up":
        pairs = [workloads.ffn_up()]
    elif name == "attn":
        pairs = [workloads.attn_proj()]
    elif name == "tiny":
        pairs = [workloads.tiny()]
    elif name == "dense_layer":
        pairs = [(A, B) for (_, A, B) in workloads.dense_layer(0)]
    elif name == "dense_request":   # the whole audited request: 32 layers x 7 matmuls, one chained transcript
        pairs = [(A, B) for layer in range(32) for (_, A, B) in workloads.dense_layer(layer)]
    elif name == "moe":
        X, routes = workloads.moe_activations()
        pairs = [(np.ascontiguousarray(X[routes[e]]), workloads.moe_expert_weight(e)) for e in range(8)]
    else:
        raise SystemExit("unknown workload %r" % name)
    out = []
    for A, B in pairs:
        Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        C = (Ad.double() @ Bd.double()).round().to(torch.int64).cpu().numpy()   # exact: |C| < 2^36
        com = imm.imm_commit_matmul(A, B, np.ascontiguousarray(C), A.shape[0], A.shape[1], B.shape[1])
        out.append((A, B, Ad, Bd, com))
    return out


def timed_runs(torch, batch, steps, warmup):
    """Milliseconds per call of batch.run(), wall clock around `steps` calls bracketed by device syncs."""
    for _ in range(warmup):
        batch.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        batch.run()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def other_workload(name, torch, imm, workloads, ctx, steps, cpu_seconds):
    """A multi-statement workload measured in the same run: the seven chained statements of one decoder
    layer (`dense_layer`) or the eight independent experts (`moe`), in the three execution modes, with
    the bandwidth of the dominant kernel (the reduction over B's columns, all statements together),
    the oracle timed on the same statements and the proofs of all modes compared with the oracle's."""
    import numpy as np
    stmts = make_workload(name, torch, imm, workloads)
    items = [(Ad, Bd, com) for (_, _, Ad, Bd, com) in stmts]
    chained = name != "moe"
    s0 = imm.imm_fs_init()
    batch = ctx.prepare_batch(items, chained, s0)
    timed_runs(torch, batch, 2, 1)
    ctx.imm_ctx_reset_profiling()
    ctx.imm_ctx_set_profiling(1 << imm.IMM_K_REDUCE_B)
    ms = timed_runs(torch, batch, steps, 0)
    ctx.imm_ctx_set_profiling(0)
    n_dom, ms_dom = ctx.imm_ctx_kernel_time(imm.IMM_K_REDUCE_B)
    ctx.imm_ctx_reset_profiling()
    proofs = [p.words() for p in batch.proofs]
    b_bytes = 8.0 * sum(B.shape[0] * B.shape[1] for (_, B, _, _, _) in stmts)
    def with_default_tail(b):
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)
        t = timed_runs(torch, b, steps, 2)
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, 0)
        return t
    ms_default = with_default_tail(batch)
    pre = [(Ad, ctx.imm_encode(Bd), com) for (Ad, Bd, com) in items]
    batch_pre = ctx.prepare_batch(pre, chained, s0)
    ms_pre = timed_runs(torch, batch_pre, steps, 2)
    proofs_pre = [p.words() for p in batch_pre.proofs]
    ms_pre_default = with_default_tail(batch_pre)
    del pre, batch_pre
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
    ms_narrow = timed_runs(torch, batch, steps, 2)
    proofs_narrow = [p.words() for p in batch.proofs]
    ms_narrow_default = with_default_tail(batch)
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
    out = {"statements": [{"m": A.shape[0], "d": A.shape[1], "n": B.shape[1]} for (A, B, _, _, _) in stmts],
           "transcript": "one chained transcript" if chained else "independent (each from the initial state)",
           "prove_ms": round(ms, 4), "prove_ms_weights_preencoded": round(ms_pre, 4),
           "prove_ms_narrow_read": round(ms_narrow, 4),
           "library_default": {"prove_ms": round(ms_default, 4), "prove_ms_weights_preencoded": round(ms_pre_default, 4),
                               "prove_ms_narrow_read": round(ms_narrow_default, 4)},
           "reduce_B": {"launches_per_step": n_dom / steps, "us_per_step": round(ms_dom * 1e3 / steps, 1),
                        "algorithmic_MB": b_bytes / 1e6,
                        "frac_of_8TBps": round(b_bytes * steps / (ms_dom * 1e-3) / 1e9 / HBM_PEAK_GBS, 3) if ms_dom else None}}
    if cpu_seconds > 0:
        from oracle import fast as oracle_fast
        from oracle import reference as ref
        oracle_items = [(A, B, None, com.digests()) for (A, B, _, _, com) in stmts]
        want, _ = oracle_fast.prove_chain(oracle_items, chained, check=False)
        want = [ref.proof_words(p) for p in want]
        n_cpu, t0 = 0, time.perf_counter()
        while n_cpu == 0 or time.perf_counter() - t0 < cpu_seconds:
            oracle_fast.prove_chain(oracle_items, chained, check=False)
            n_cpu += 1
        out["cpu_baseline"] = {"value": round((time.perf_counter() - t0) * 1e3 / n_cpu, 2), "unit": "ms",
                               "cores": oracle_fast.threads(), "kind": "oracle", "sample": ORACLE_FORM % n_cpu}
        out["proof_bytes_equal"] = bool(proofs == want and proofs_pre == want and proofs_narrow == want)
    return out


ORACLE_FORM = ("the full workload (same statements), %d repetitions; the oracle's prove with c0 taken as sum_j a[j] b[j] "
               "like the prover's (C=None, check=False: the product matrix is not read, no direct openings)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="ffn_up", choices=["ffn_up", "attn", "tiny", "dense_layer", "dense_request", "moe"],
                    help="dense_request (224 chained proofs) wants --steps 3 --warmup 1")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="time budget of the CPU-oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the decoder-layer and expert-batch workloads that the default run (ffn_up) also measures")
    ap.add_argument("--fold-log2", type=int, default=26,
                    help="log2 of the table length of the stand-alone fold-kernel measurement (0 = skip)")
    ap.add_argument("--ldd-steps", type=int, default=2048,
                    help="decision steps of the logit-distance measurement (vocabulary 128256, K = 20); 0 skips it")
    ap.add_argument("--timeline", action="store_true",
                    help="after the timed region, prove the first statement 20 more times in each execution mode with the "
                         "library's host-side time marks switched on and report them (field host_timeline): medians in "
                         "microseconds from the call's entry, and the absolute CLOCK_MONOTONIC marks of the last proof "
                         "for lining up with a rocprofv3 kernel trace of the same run")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 512 MiB device copy three times (reference dispatches for scaling "
                         "hardware byte counters collected with rocprofv3 --pmc)")
    ap.add_argument("--narrow", action="store_true",
                    help="skip the encoding pass: the reductions read int8/int16 directly (reported as an extra "
                         "field by default; with this flag it becomes the timed path)")
    ap.add_argument("--transcript", default="host", choices=["device", "host"],
                    help="who hashes the round messages: lane 0 of the round kernel, or the host via the mailbox")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU only: the prover path has no multi-GPU part "
                         "(run with --gpus 1)")

    import torch
    from paper_2602_22700_amd import binding as imm
    from paper_2602_22700_amd import workloads

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    imm.load()
    stmts = make_workload(args.workload, torch, imm, workloads)
    ctx = imm.Context(0)
    ctx.imm_ctx_set_option(imm.IMM_OPT_TRANSCRIPT,
                           imm.IMM_TRANSCRIPT_HOST if args.transcript == "host" else imm.IMM_TRANSCRIPT_DEVICE)
    if args.narrow:
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
    # What is timed as `value` (and every prove_ms* beside it) runs every step of the path in the kernels:
    # all rounds of the sumcheck on the device.  The library's default hands the rounds on tables of at
    # most 512 entries to the calling thread, which is faster; those figures are under "library_default".
    ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, 0)
    items = [(Ad, Bd, com) for (_, _, Ad, Bd, com) in stmts]
    chained = len(items) > 1 and args.workload != "moe"   # experts are independent statements
    s0 = imm.imm_fs_init()

    batch = ctx.prepare_batch(items, chained, s0)   # arguments marshalled once; a step is one C call
    step = batch.run

    for _ in range(args.warmup):
        step()
    dominant = imm.IMM_K_REDUCE_B
    ctx.imm_ctx_reset_profiling()
    ctx.imm_ctx_set_profiling(1 << dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    proofs = batch.proofs
    ctx.imm_ctx_set_profiling(0)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_dom, ms_dom = ctx.imm_ctx_kernel_time(dominant)

    # per-kernel breakdown in a separate, untimed pass (events around every kernel)
    ctx.imm_ctx_reset_profiling()
    ctx.imm_ctx_set_profiling((1 << imm.IMM_K_COUNT) - 1)
    reps = max(3, min(10, args.steps))
    for _ in range(reps):
        step()
    ctx.imm_ctx_set_profiling(0)
    kernels = {}
    for k in range(imm.IMM_K_COUNT):
        n, ms = ctx.imm_ctx_kernel_time(k)
        kernels[imm.KERNEL_NAMES[k]] = {"launches_per_step": n / reps, "us_per_step": round(ms * 1e3 / reps, 2)}

    # algorithmic bytes of the dominant kernel: 8 B per entry of every B streamed in one step, plus
    # 8 B per entry of A where both reductions share a launch (then no launch is booked under reduce_A)
    b_entries = sum(B.shape[0] * B.shape[1] for (_, B, _, _, _) in stmts)
    a_entries = sum(A.shape[0] * A.shape[1] for (A, _, _, _, _) in stmts)
    fused = kernels["reduce_A"]["launches_per_step"] == 0
    dom_bytes = 8.0 * b_entries + (8.0 * a_entries if fused else 0.0)
    launches_per_step = n_dom / args.steps
    avg_ms = ms_dom / max(n_dom, 1)
    achieved = (dom_bytes / launches_per_step) / (avg_ms * 1e-3) / 1e9 if n_dom else 0.0
    # where the widening of A and B and the eq vectors share a launch it is booked under encode_B
    front = kernels["encode_A"]["launches_per_step"] == 0 and kernels["encode_B"]["launches_per_step"] > 0
    for name, nbytes in (("encode_A", 0 if front else 10 * a_entries),
                         ("encode_B", 9 * b_entries + (10 * a_entries if front else 0)),
                         ("reduce_A", 0 if fused else 8 * a_entries), ("reduce_B", dom_bytes)):
        us = kernels[name]["us_per_step"]
        if not nbytes:
            continue
        kernels[name]["algorithmic_MB"] = round(nbytes / 1e6, 1)
        kernels[name]["GBps"] = round(nbytes / (us * 1e-6) / 1e9, 1) if us else None
        kernels[name]["frac_of_8TBps"] = round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 3) if us else None
    if fused:
        kernels["reduce_B"]["covers"] = "reduce_A and reduce_B in one launch"
    if front:
        kernels["encode_B"]["covers"] = "encode_A, encode_B and eq_build in one launch"
    if kernels["combine"]["launches_per_step"] == 0 and not fused:
        kernels["reduce_B"]["covers"] = "reduce_B and the sum of reduce_A's partial vectors in one launch"

    def with_default_tail(b):
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, imm.IMM_HOST_TAIL_DEFAULT)
        t = timed_runs(torch, b, args.steps, 2)
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, 0)
        return t
    ms_default = with_default_tail(batch)

    # the same step with the weights widened beforehand (deployment-time encoding)
    items_pre = [(Ad, ctx.imm_encode(Bd), com) for (Ad, Bd, com) in items]
    batch_pre = ctx.prepare_batch(items_pre, chained, s0)
    ms_pre = timed_runs(torch, batch_pre, args.steps, 2)
    pre_proofs = batch_pre.proofs
    ms_pre_default = with_default_tail(batch_pre)
    # ... and the activations read as they are stored (no widening at all inside the call)
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
    ms_pre_raw = timed_runs(torch, batch_pre, args.steps, 2)
    pre_raw_proofs = batch_pre.proofs
    ms_pre_raw_default = with_default_tail(batch_pre)
    ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0 if args.narrow else 1)
    del items_pre, batch_pre

    ms_narrow, narrow_proofs, ms_narrow_default = None, None, None
    if not args.narrow:
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 0)
        ms_narrow = timed_runs(torch, batch, args.steps, 2)
        narrow_proofs = batch.proofs
        ms_narrow_default = with_default_tail(batch)
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)

    result = {
        "metric": "matmul_sumcheck_prove_time_per_layer", "value": round(ms_per_step, 4), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u64 (Goldilocks field)",
        "data": "synthetic",
        "value_is": ("ms for the proofs of this workload's statements (%d matrix product%s = %d linear layer%s of the model)"
                     % (len(stmts), "" if len(stmts) == 1 else "s", len(stmts), "" if len(stmts) == 1 else "s")
                     + ("; a decoder layer of seven is other_workloads.dense_layer" if args.workload == "ffn_up" else "")),
        "config": {"workload": args.workload,
                   "statements": ([{"m": A.shape[0], "d": A.shape[1], "n": B.shape[1]} for (A, B, _, _, _) in stmts]
                                  if len(stmts) <= 8 else "%d chained statements: 32 decoder layers x (Wq, Wk, Wv, Wo, "
                                  "W_gate, W_up, W_down), 1024 tokens" % len(stmts)),
                   "A": "int16 Gaussian sigma=2^10", "B": "int8 uniform", "transcript": "SHA-256 Fiat-Shamir, hashed on the " + args.transcript,
                   "includes": ("eq, narrow-read reduce A+B, rounds, hashing" if args.narrow
                                else "encode A+B, eq, reduce A+B, rounds, hashing")},
        "prove_ms_weights_preencoded": round(ms_pre, 4),
        "prove_ms_weights_preencoded_activations_read_raw": round(ms_pre_raw, 4),
        "prove_ms_narrow_read": round(ms_narrow, 4) if ms_narrow is not None else None,
        "rounds": "every round of the sumcheck on the device (IMM_OPT_HOST_TAIL = 0) in value, in the prove_ms_* beside it, in "
                  "kernels and in other_workloads; library_default holds the same measurements with the library's default, in "
                  "which the calling thread, which hashes every round's message anyway, finishes the rounds on tables of at "
                  "most 512 entries",
        "library_default": {"prove_ms": round(ms_default, 4), "prove_ms_weights_preencoded": round(ms_pre_default, 4),
                            "prove_ms_weights_preencoded_activations_read_raw": round(ms_pre_raw_default, 4),
                            "prove_ms_narrow_read": round(ms_narrow_default, 4) if ms_narrow_default is not None else None},
        "kernels": kernels,
        "roofline": {"bound": "hbm",
                     "kernel": ("reduce_A+B (partial MLEs of A over its rows and of B over its columns, one launch)" if fused
                                else "reduce_B (partial MLE of B over its columns)" +
                                ("; the launch also sums the partial vectors of A's reduction, whose bytes are not counted"
                                 if kernels["combine"]["launches_per_step"] == 0 else "")),
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": recorded_traffic() if args.workload == "ffn_up" else None,
                     "traffic_source": "profiles/reduce_B_ffn_up_hbm_counters.txt (recorded with rocprofv3 --pmc in an earlier "
                                       "run of this command, not measured in this run; null once the kernel sources differ)",
                     "avg_launch_us": round(avg_ms * 1e3, 2), "algorithmic_bytes_per_launch": dom_bytes / max(launches_per_step, 1)},
    }

    if args.timeline:
        import statistics
        Ad0, Bd0, com0 = items[0]
        Bpre0 = ctx.imm_encode(Bd0)
        ctx.imm_ctx_set_option(imm.IMM_OPT_TIMELINE, 1)
        tl = {}
        for mode, Bx, widen, tail in (("widened", Bd0, 1, 0), ("weights_preencoded", Bpre0, 1, 0), ("narrow_read", Bd0, 0, 0),
                                      ("widened, library default", Bd0, 1, imm.IMM_HOST_TAIL_DEFAULT),
                                      ("weights_preencoded, library default", Bpre0, 1, imm.IMM_HOST_TAIL_DEFAULT),
                                      ("narrow_read, library default", Bd0, 0, imm.IMM_HOST_TAIL_DEFAULT)):
            ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, widen)
            ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, tail)
            runs = []
            for _ in range(23):
                ctx.imm_sumcheck_matmul_prove(Ad0, Bx, com0, s0)
                runs.append(ctx.imm_debug_timeline())
            runs = runs[3:]
            names = [nm for nm, _ in runs[-1]]
            tl[mode] = {"us_from_entry_median": {nm: round(statistics.median((r[i][1] - r[0][1]) / 1e3 for r in runs), 2)
                                                 for i, nm in enumerate(names)},
                        "last_proof_monotonic_ns": {nm: t for nm, t in runs[-1]}}
        ctx.imm_ctx_set_option(imm.IMM_OPT_WIDEN, 1)
        ctx.imm_ctx_set_option(imm.IMM_OPT_HOST_TAIL, 0)
        ctx.imm_ctx_set_option(imm.IMM_OPT_TIMELINE, 0)
        result["host_timeline"] = tl
        del Bpre0

    # Opening of C at (rx || ry): the bilinear MLE of the int64 product matrix, streamed once by the
    # same row-wise reduction (8 B per entry), as a verifier-side check would need it.
    if args.workload == "ffn_up":
        A0, B0 = stmts[0][2], stmts[0][3]
        Cd = (A0.double() @ B0.double()).round().to(torch.int64)
        pr = [(0x9E3779B97F4A7C15 * (i + 1)) % 0xFFFFFFFF00000001 for i in range(11)]
        pc = [(0xC2B2AE3D27D4EB4F * (i + 1)) % 0xFFFFFFFF00000001 for i in range(14)]
        for _ in range(2):
            ctx.imm_mle_eval(Cd, pr, pc)
        ctx.imm_ctx_reset_profiling()
        ctx.imm_ctx_set_profiling(1 << imm.IMM_K_REDUCE_B)
        for _ in range(10):
            ctx.imm_mle_eval(Cd, pr, pc)
        ctx.imm_ctx_set_profiling(0)
        nc, msc = ctx.imm_ctx_kernel_time(imm.IMM_K_REDUCE_B)
        usc = msc * 1e3 / nc
        cbytes = Cd.numel() * 8
        result["mle_eval_C_int64"] = {"rows": Cd.shape[0], "cols": Cd.shape[1], "us_per_launch": round(usc, 1),
                                      "algorithmic_MB": cbytes / 1e6, "GBps": round(cbytes / (usc * 1e-6) / 1e9, 1),
                                      "frac_of_8TBps": round(cbytes / (usc * 1e-6) / 1e9 / HBM_PEAK_GBS, 3)}
        ctx.imm_ctx_reset_profiling()

        # Commitments of the statement's activations and product hashed where they live: one lane per
        # 1 MiB leaf, so the launch time is that of one leaf's hash chain, here and for up to 65536 leaves.
        Cc = Cd.contiguous()
        tabs = [A0, Cc]
        got = ctx.imm_commit_tables_device(tabs)
        t0 = time.perf_counter()
        for _ in range(3):
            got = ctx.imm_commit_tables_device(tabs)
        dev_ms = (time.perf_counter() - t0) * 1e3 / 3
        Ah, Ch = A0.cpu().numpy(), Cc.cpu().numpy()
        host = imm.imm_commit_matmul(Ah, None, Ch, Ah.shape[0], Ah.shape[1], Ch.shape[1])
        t0 = time.perf_counter()
        for _ in range(3):
            host = imm.imm_commit_matmul(Ah, None, Ch, Ah.shape[0], Ah.shape[1], Ch.shape[1])
        host_ms = (time.perf_counter() - t0) * 1e3 / 3
        nbytes = A0.numel() * 2 + Cc.numel() * 8
        result["commit_A_and_C"] = {"leaves": sum((t.numel() * t.element_size() + (1 << 20) - 1) >> 20 for t in tabs),
                                    "MB": nbytes / 1e6, "device_ms": round(dev_ms, 2), "host_ms": round(host_ms, 2),
                                    "host_threads": min(16, os.cpu_count() or 1),
                                    "same_digests": [bytes(g.digest) for g in got] == [bytes(host.A.digest), bytes(host.C.digest)]}
        del Cd, Cc, Ah, Ch

    # The per-round kernel on tables large enough to be bandwidth-bound (the proof's own tables are
    # 2 x 32 KB, i.e. latency-bound): fold + evaluate on two tables of 2^26 elements, in place.
    # Algorithmic bytes per launch: 16 B read + 8 B written per table entry pair = 24 * L.
    if args.fold_log2 > 0:
        Lf = 1 << args.fold_log2
        ta = torch.randint(0, 1 << 62, (Lf,), dtype=torch.int64, device="cuda").view(torch.uint64)
        tb = torch.randint(0, 1 << 62, (Lf,), dtype=torch.int64, device="cuda").view(torch.uint64)
        for _ in range(2):
            ctx.imm_round_fold_eval(ta, tb, Lf, fold_r=0x123456789ABCDEF)
        ctx.imm_ctx_reset_profiling()
        ctx.imm_ctx_set_profiling(1 << imm.IMM_K_ROUND)
        for _ in range(10):
            ctx.imm_round_fold_eval(ta, tb, Lf, fold_r=0x123456789ABCDEF)
        ctx.imm_ctx_set_profiling(0)
        nf, msf = ctx.imm_ctx_kernel_time(imm.IMM_K_ROUND)
        us = msf * 1e3 / nf
        result["fold_kernel_large_tables"] = {"L": Lf, "us_per_launch": round(us, 1), "algorithmic_MB": 24 * Lf / 1e6,
                                              "GBps": round(24 * Lf / (us * 1e-6) / 1e9, 1),
                                              "frac_of_8TBps": round(24 * Lf / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 3),
                                              "traffic_mix": "2 bytes read per byte written, in place"}
        ctx.imm_ctx_reset_profiling()
        del ta, tb

    # The reduction of A over its rows (K3a) on a table large enough for its launch to be mostly
    # streaming: 16384 x 4096 field elements (537 MB), as the A of a statement with a narrow B, both
    # operands passed pre-encoded and each reduction in a launch of its own.  At the FFN shape the same
    # kernel reads 67 MB in a launch that is largely filling and draining the machine.
    if args.workload == "ffn_up":
        mL, dL, nL = 16384, 4096, 16
        Al = torch.randint(0, 1 << 62, (mL, dL), dtype=torch.int64, device="cuda").view(torch.uint64)
        Bl = torch.randint(0, 1 << 62, (dL, nL), dtype=torch.int64, device="cuda").view(torch.uint64)
        zA, zB, zC = (torch.zeros(sh, dtype=dt).numpy() for sh, dt in (((1, 1), torch.int16), ((1, 1), torch.int8), ((1, 1), torch.int64)))
        comL = imm.imm_commit_matmul(zA, zB, zC, 1, 1, 1)      # digests of anything: the prover only absorbs them
        for c1, rows, cols in ((comL.A, mL, dL), (comL.B, dL, nL), (comL.C, mL, nL)):
            c1.rows, c1.cols = rows, cols
        ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 0)
        for _ in range(2):
            ctx.imm_sumcheck_matmul_prove(Al, Bl, comL, s0)
        ctx.imm_ctx_reset_profiling()
        ctx.imm_ctx_set_profiling(1 << imm.IMM_K_REDUCE_A)
        for _ in range(10):
            ctx.imm_sumcheck_matmul_prove(Al, Bl, comL, s0)
        ctx.imm_ctx_set_profiling(0)
        ctx.imm_ctx_set_option(imm.IMM_OPT_FUSE_REDUCTIONS, 1)
        na, msa = ctx.imm_ctx_kernel_time(imm.IMM_K_REDUCE_A)
        usa = msa * 1e3 / na
        abytes = 8 * mL * dL
        result["reduce_A_large"] = {"rows": mL, "cols": dL, "us_per_launch": round(usa, 1), "algorithmic_MB": abytes / 1e6,
                                    "GBps": round(abytes / (usa * 1e-6) / 1e9, 1),
                                    "frac_of_8TBps": round(abytes / (usa * 1e-6) / 1e9 / HBM_PEAK_GBS, 3)}
        ctx.imm_ctx_reset_profiling()
        del Al, Bl

    # What the memory system of this machine delivers to plain library kernels with the same traffic mixes
    # (512 MiB operands, HIP events on torch's stream): the practical ceilings next to the 8 TB/s peak.
    if args.workload == "ffn_up":
        nel = 64 << 20
        u = torch.arange(nel, dtype=torch.int64, device="cuda")
        v = torch.ones(nel, dtype=torch.int64, device="cuda")
        o = torch.empty(nel, dtype=torch.int64, device="cuda")

        def torch_rate(fn, nbytes, reps=10):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            e1.synchronize()
            return round(nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

        result["memory_ceilings_GBps"] = {
            "read_only (torch.sum, 512 MiB)": torch_rate(lambda: u.sum(), 8 * nel),
            "write_only (fill_, 512 MiB)": torch_rate(lambda: o.fill_(7), 8 * nel),
            "copy 1 read : 1 write (copy_, 2 x 512 MiB)": torch_rate(lambda: o.copy_(u), 16 * nel),
            "2 reads : 1 write (torch.add out=, 3 x 512 MiB)": torch_rate(lambda: torch.add(u, v, out=o), 24 * nel),
            "note": "library kernels of the PyTorch build in this image, not tuned for this part; the hand-written "
                    "kernels above are to be read against the 8 TB/s peak, these only say what a plain stream gets"}
        del u, v, o

    # The logit-distance step of the audit on the logits of `ldd_steps` decision steps over a
    # 128256-entry vocabulary: TV and KL of the two softmax rows (8 B per vocabulary entry: one fp32
    # logit of each model) and the top-K distance of the deployed row (4 B per entry), K = 20.
    if args.ldd_steps > 0:
        Tl, nl, Kl = args.ldd_steps, 128256, 20
        dep_h, ref_h = workloads.logits_pair(Tl, nl, seed=2025)
        idx_h = workloads.topk_indices(dep_h, Kl)
        dep_d, ref_d, idx_d = torch.from_numpy(dep_h).cuda(), torch.from_numpy(ref_h).cuda(), torch.from_numpy(idx_h).cuda()

        def timed(kid, fn, reps=20):
            for _ in range(3):
                fn()
            ctx.imm_ctx_reset_profiling()
            ctx.imm_ctx_set_profiling(1 << kid)
            for _ in range(reps):
                fn()
            ctx.imm_ctx_set_profiling(0)
            nk, msk = ctx.imm_ctx_kernel_time(kid)
            ctx.imm_ctx_reset_profiling()
            return msk * 1e3 / nk

        def line(us, nbytes):
            return {"us_per_launch": round(us, 1), "algorithmic_MB": nbytes / 1e6,
                    "GBps": round(nbytes / (us * 1e-6) / 1e9, 1),
                    "frac_of_8TBps": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 3)}

        ldd = {"steps": Tl, "vocab": nl, "K": Kl, "dtype": "f32 logits, f64 sums"}
        ldd["tv_and_kl"] = line(timed(imm.IMM_K_LDD, lambda: ctx.imm_ldd_tv_kl(dep_d, ref_d)), 8 * Tl * nl)
        ldd["kl_only"] = line(timed(imm.IMM_K_LDD, lambda: ctx.imm_ldd_tv_kl(dep_d, ref_d, want_tv=False)), 8 * Tl * nl)
        ldd["topk_distance"] = line(timed(imm.IMM_K_TOPK, lambda: ctx.imm_topk_distance(dep_d, idx_d)), 4 * Tl * nl)
        if not args.no_cpu_baseline:
            from oracle import ldd as oracle_ldd
            rows = list(range(0, Tl, max(1, Tl // 16)))[:16]
            t0 = time.perf_counter()
            for i in rows:
                oracle_ldd.tv_distance(dep_h[i], ref_h[i])
                oracle_ldd.kl_divergence(dep_h[i], ref_h[i])
            t1 = time.perf_counter()
            for i in rows:
                oracle_ldd.topk_distance(dep_h[i], idx_h[i])
            t2 = time.perf_counter()
            ldd["cpu_oracle"] = {"tv_and_kl_ms_per_step": round((t1 - t0) * 1e3 / len(rows), 2),
                                 "topk_ms_per_step": round((t2 - t1) * 1e3 / len(rows), 2), "cores": 1,
                                 "sample": "%d of the %d steps" % (len(rows), Tl)}
        result["logit_distance"] = ldd
        del dep_d, ref_d, idx_d, dep_h, ref_h

    # All activations and products of the audited request committed in one launch (synthetic bytes of
    # the real sizes: a hash does not care), which is the case the device-side leaf hashing is for.
    if args.workload == "dense_request":
        tabs = []
        for (A, B, _, _, _) in stmts:
            tabs.append(torch.randint(-2**15, 2**15, A.shape, dtype=torch.int16, device="cuda"))
            tabs.append(torch.randint(-2**40, 2**40, (A.shape[0], B.shape[1]), dtype=torch.int64, device="cuda"))
        ctx.imm_commit_tables_device(tabs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2):
            ctx.imm_commit_tables_device(tabs)
        dev_ms = (time.perf_counter() - t0) * 1e3 / 2
        nbytes = sum(t.numel() * t.element_size() for t in tabs)
        sample = [t.cpu().numpy() for t in tabs[:14]]     # the first layer, on the host
        t0 = time.perf_counter()
        for k in range(0, 14, 2):
            imm.imm_commit_matmul(sample[k], None, sample[k + 1], sample[k].shape[0], sample[k].shape[1], sample[k + 1].shape[1])
        host_layer_ms = (time.perf_counter() - t0) * 1e3
        # the same commitments (as the next request's would be) while this request is being proven: a
        # second context and stream, driven by a second host thread
        import threading
        ctx2 = imm.Context(0)
        side = torch.cuda.Stream()
        ctx2.imm_commit_tables_device(tabs, stream=side)
        both = []
        for _ in range(2):
            th = threading.Thread(target=lambda: ctx2.imm_commit_tables_device(tabs, stream=side))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            th.start()
            step()
            th.join()
            torch.cuda.synchronize()
            both.append((time.perf_counter() - t0) * 1e3)
        ctx2.close()
        result["commit_A_and_C_of_the_request"] = {
            "tables": len(tabs), "leaves": sum((t.numel() * t.element_size() + (1 << 20) - 1) >> 20 for t in tabs),
            "GB": round(nbytes / 1e9, 2), "device_ms": round(dev_ms, 1), "device_GBps": round(nbytes / dev_ms / 1e6, 1),
            "prove_and_commit_side_by_side_ms": round(min(both), 1),
            "host_ms_extrapolated": round(host_layer_ms * len(stmts) / 7, 1),
            "host_sample": "the 7 statements of one layer, %d threads" % min(16, os.cpu_count() or 1)}
        del tabs, sample

    if args.calibrate_copy:
        src = torch.arange(64 << 20, dtype=torch.int64, device="cuda")   # 512 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibration_copy_bytes_each_way"] = src.numel() * 8
        del src, dst

    if not args.no_cpu_baseline:
        from oracle import fast as oracle_fast
        from oracle import reference as ref
        oracle_items = [(A, B, None, com.digests()) for (A, B, _, _, com) in stmts]
        want, _ = oracle_fast.prove_chain(oracle_items, chained, check=False)   # also warms the library
        same = [p.words() for p in proofs] == [ref.proof_words(p) for p in want] and \
               [p.words() for p in pre_proofs] == [ref.proof_words(p) for p in want] and \
               [p.words() for p in pre_raw_proofs] == [ref.proof_words(p) for p in want] and \
               (narrow_proofs is None or [p.words() for p in narrow_proofs] == [ref.proof_words(p) for p in want])
        n_cpu, t_cpu0 = 0, time.perf_counter()
        while True:
            oracle_fast.prove_chain(oracle_items, chained, check=False)
            n_cpu += 1
            if time.perf_counter() - t_cpu0 >= args.cpu_seconds:
                break
        cpu_ms = (time.perf_counter() - t_cpu0) * 1e3 / n_cpu
        result["cpu_baseline"] = {"value": round(cpu_ms, 2), "unit": "ms", "cores": oracle_fast.threads(),
                                  "kind": "oracle", "sample": ORACLE_FORM % n_cpu}
        result["proof_bytes_equal"] = bool(same)

    # The multi-statement workloads of the metric (ms per layer): one decoder layer and the expert batch.
    if args.workload == "ffn_up" and not args.no_other_workloads:
        del stmts, items, batch, step
        torch.cuda.empty_cache()
        result["other_workloads"] = {
            name: other_workload(name, torch, imm, workloads, ctx, 10, 0.0 if args.no_cpu_baseline else 3.0)
            for name in ("dense_layer", "moe")}
    # the other kernels the bandwidth target names, next to the dominant one
    also = {}
    if "frac_of_8TBps" in kernels.get("reduce_A", {}):
        also["reduce_A (K3a) at this shape"] = kernels["reduce_A"]["frac_of_8TBps"]
    if "reduce_A_large" in result:
        also["reduce_A (K3a) on 16384 x 4096"] = result["reduce_A_large"]["frac_of_8TBps"]
    if "fold_kernel_large_tables" in result:
        also["fold + evaluate (K4) on 2^%d entries" % args.fold_log2] = result["fold_kernel_large_tables"]["frac_of_8TBps"]
    if "frac_of_8TBps" in kernels.get("encode_B", {}):
        also["encode (K1, with K2 where they share a launch)"] = kernels["encode_B"]["frac_of_8TBps"]
    result["roofline"]["other_streaming_kernels_frac"] = also
    print(json.dumps(result))


if __name__ == "__main__":
    main()
