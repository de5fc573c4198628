"""Benchmark of the Pacer hot path on one MI355X.

One "step" is one outer iteration of Alg. 1 through the four hot calls (b x draft_step +
preverify_block per round, verify, accept_rollback) on the 7B/68M-shaped synthetic pair:
512-token uniform-random prompt, stochastic sampling at temperature 1, gamma_max 16, b 4, beta 3.
Prints ONE JSON line (see the fields at the bottom).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0   # dense f16/bf16 matrix peak of MI355X


def weight_bytes(shape, n_layers=None):
    d, f, v = shape["d_model"], shape["d_ffn"], shape["vocab"]
    L = shape["n_layers"] if n_layers is None else n_layers
    return 2.0 * (L * (4 * d * d + 3 * d * f) + v * d)


def run_steps(sess, n, mode, seed, batch=None, **kw):
    """n outer iterations of Alg. 1 (for a batch: n lock-step iterations of all sequences)."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    toks, gam, acc, cnt = 0, 0, 0, 0
    reached, accepted = [0] * 32, [0] * 32            # per draft position 1..gamma_max
    for _ in range(n):
        if batch is None:
            rs = [sess.step(mode=mode, seed=seed, **kw)]
        else:
            rs = sess.step_batch(batch["seqs"], mode=mode, betas=batch["betas"], seed=seed, **kw)
        for r in rs:
            toks += r["n"] + 1
            gam += r["gamma"]
            acc += r["n"]
            cnt += 1
            for i in range(r["gamma"]):               # position i+1 is tested iff the i before it were accepted
                if r["n"] >= i:
                    reached[i] += 1
                    accepted[i] += 1 if r["n"] > i else 0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dict(tokens=toks, seconds=dt, tok_s=toks / dt, ms_per_step=1e3 * dt / max(n, 1),
                mean_gamma=gam / max(cnt, 1), tau=acc / max(cnt, 1), reached=reached, accepted=accepted)


def cpu_baseline(w, tgt, drf, mb, prompt, mode, budget_s=10.0, threads=None):
    """The CPU oracle as it stands, on the host cores, on a bounded sample of the same workload: the
    workload's full prompt (untimed, as on the GPU), then decoding steps (timed) until the workload's number of
    new tokens is reached (the small workloads run in full) or `budget_s` seconds have passed, two steps at least."""
    import numpy as np
    import helpers
    from threadpoolctl import threadpool_info, threadpool_limits
    ctl = threadpool_limits(limits=threads) if threads else None
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    want = int(w["new"])
    o = helpers.build_oracle(w, tgt, drf, mb, mode=mode, seed=3, max_seq=len(prompt) + want + w["gamma_max"] + 64)
    t0 = time.perf_counter()
    o.prefill(prompt)
    t_prompt = time.perf_counter() - t0
    t0 = time.perf_counter()
    toks = steps = 0
    while True:
        r = o.step()
        toks += r["n"] + 1
        steps += 1
        dt = time.perf_counter() - t0
        if toks >= want or (steps >= 2 and dt >= budget_s):
            break
    if ctl is not None:
        ctl.restore_original_limits()
    full = "the workload's full decode" if toks >= want else "a bounded sample"
    return {"value": toks / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{steps} Pacer decoding steps ({toks} tokens, {dt:.1f} s, timed; {full}) of the same pair after the "
                      f"workload's full {len(prompt)}-token prompt ({t_prompt:.1f} s, untimed); numpy float64 oracle, "
                      f"{int(cores)} BLAS thread{'s' if cores != 1 else ''}"}


def stream_ceiling(torch, B, shape=None, n_layers=None):
    """What this GPU delivers to kernels that only move data: a streaming read (the library's probe kernel) and a
    plain device-to-device copy of 2 GiB, in GB/s (the copy counts read + written bytes)."""
    n = 1 << 31
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = 1e30
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best
    read_ms = timed(lambda: B.pacer_stream_probe(src, sink, st))
    copy_ms = timed(lambda: dst.copy_(src))
    # The same probe as ONE launch of the size of each of the target's matrices, in a chain of launches over
    # consecutive cold regions (as the GEMMs of a verify pass follow each other): the time a kernel needs that
    # does nothing but read those bytes, launch and ramp included.  Their sum over a pass is the floor of any
    # design with one launch per matrix.
    floors = None
    if shape is not None:
        d, f, v = shape["d_model"], shape["d_ffn"], shape["vocab"]
        L = shape["n_layers"] if n_layers is None else n_layers
        sizes = {"qkv": 3 * d * d * 2, "o": d * d * 2, "gate_up": 2 * f * d * 2, "down": d * f * 2, "lm_head": v * d * 2}
        floors = {}
        for name, nb in sizes.items():
            nb = nb // 4096 * 4096
            reps = max(2, min(24, n // nb))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            best = 1e30
            for _ in range(3):
                torch.cuda.synchronize()
                e0.record()
                for r in range(reps):
                    B.pacer_stream_probe(src[r * nb:(r + 1) * nb], sink, st)
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
            floors[name] = {"MB": round(nb / 1e6, 1), "us": round(best, 2)}
        per_layer = sum(floors[k]["us"] for k in ("qkv", "o", "gate_up", "down"))
        floors["pass_ms_without_attention"] = round((L * per_layer + floors["lm_head"]["us"]) / 1e3, 4)
    # 1000 launches that read 4 KiB each, enqueued back to back by the library: what one more kernel in a sequence
    # of launches costs when it does next to nothing (the floor under each of the 13 launches of a draft step)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tiny = 1e30
    for _ in range(3):
        torch.cuda.synchronize()
        e0.record()
        B.pacer_stream_probe(src[:4096], sink, st, repeat=1000)
        e1.record()
        torch.cuda.synchronize()
        tiny = min(tiny, e0.elapsed_time(e1) * 1e3 / 1000)
    del src, dst
    torch.cuda.empty_cache()
    return {"streaming_read_GBps": round(n / 1e6 / read_ms, 1), "device_copy_GBps": round(2 * n / 1e6 / copy_ms, 1),
            "bytes": n, "per_launch_read_floor": floors, "empty_launch_us": round(tiny, 2), "note": "best of 5; the read kernel is the library's probe (16-byte loads, 256 blocks of 4 waves, 8 loads in flight per lane)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="7b")
    ap.add_argument("--layers", type=int, default=None, help="truncate target depth (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-one-thread", action="store_true",
                    help="also time the CPU oracle with one BLAS thread (small workloads: tiny, mid)")
    ap.add_argument("--no-context", action="store_true", help="skip the AR / fixed-gamma context runs")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for scaling rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_01274_amd import synth
    from paper_2602_01274_amd import binding as B
    from paper_2602_01274_amd.engine import Session

    torch.cuda.set_device(0)
    w = synth.workload(a.workload)
    mode = B.SAMPLE if w["mode"] == "sample" else B.GREEDY
    K, W = a.steps, a.warmup
    nb = w["batch"]
    batch = None
    if nb > 1:
        lens = synth.make_lengths(w["prompt"][0], w["prompt"][1], nb, 4)
        batch = dict(seqs=list(range(nb)), betas=synth.make_betas(1.0, 5.0, nb, 5))
        w["beta"] = sum(batch["betas"]) / nb
        n_prompt = max(lens)
    else:
        lens = [w["prompt"]]
        n_prompt = w["prompt"]
    max_seq = n_prompt + (K + W) * (w["gamma_max"] + 1) + 64
    tgt, drf, mb = synth.make_pair(w, seed=0, device="cuda", n_layers_target=a.layers)
    prompts = [synth.make_prompt(w["target"]["vocab"], n, 1 + i).tolist() for i, n in enumerate(lens)]
    prompt = prompts[0]
    sess = Session(w, tgt, drf, mb, max_seq=max_seq, max_batch=nb)
    host = None
    if not a.no_cpu_baseline:
        to_host = lambda x: ({k: to_host(v) for k, v in x.items()} if isinstance(x, dict)
                             else [to_host(v) for v in x] if isinstance(x, list) else x.cpu())
        host = (to_host(tgt), to_host(drf), to_host(mb))
    del tgt, drf, mb
    torch.cuda.empty_cache()

    def fresh():
        for i, p in enumerate(prompts):
            sess.prefill(p, seq=i)
        sess.counts = dict(draft=0, target=0, preverify=0)

    # ---- prompt ingestion (not part of the metric; reported as context) ----
    fresh()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fresh()
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) * 1e3

    # ---- the timed region: W warm-up steps, then exactly K steps ----
    run_steps(sess, W, mode, 3, batch)
    main_run = run_steps(sess, K, mode, 3, batch)
    counts = dict(sess.counts)

    # ---- same K steps with HIP events around every launch of the weight-streaming GEMM ----
    fresh()
    run_steps(sess, W, mode, 3, batch)
    B.pacer_profile_enable(sess.ctx, True)
    B.pacer_profile_read(sess.ctx)
    run_steps(sess, K, mode, 3, batch)                     # every launch of the K steps (the library holds 16384 event pairs)
    n_launch, gemm_ms, gemm_bytes = B.pacer_profile_read(sess.ctx)
    B.pacer_profile_enable(sess.ctx, False)

    # ---- per-call timing (events around each C call) ----
    fresh()
    run_steps(sess, W, mode, 3, batch)
    sess.timers = {}
    prof_steps = min(K, 40)
    run_steps(sess, prof_steps, mode, 3, batch)
    tm = sess.read_timers()
    nl = sess.read_launches()
    sess.timers = None
    L = a.layers if a.layers else w["target"]["n_layers"]
    ctx_len = sum(lens) + 0.5 * main_run["tokens"]        # summed over the batch
    kv_t = 2.0 * 2 * w["target"]["d_model"] * L * ctx_len
    kv_d = 2.0 * 2 * w["draft"]["d_model"] * w["draft"]["n_layers"] * ctx_len
    alg = {"verify": weight_bytes(w["target"], L) + kv_t,
           "draft_step": weight_bytes(w["draft"]) + kv_d,
           "preverify_block": weight_bytes(w["draft"], 1) - 2.0 * w["draft"]["vocab"] * w["draft"]["d_model"] + kv_d / w["draft"]["n_layers"]}
    calls = {}
    for name, ts in tm.items():
        ms = sum(ts) / len(ts)
        q = sorted(ts)
        pct = lambda f: q[min(len(q) - 1, int(f * len(q)))]
        calls[name] = {"mean_ms": round(ms, 4), "median_ms": round(pct(0.5), 4), "p10_ms": round(pct(0.1), 4),
                       "p90_ms": round(pct(0.9), 4), "n": len(ts),
                       "launches_per_call": round(sum(nl.get(name, [0])) / max(1, len(nl.get(name, [0]))), 2)}
        if name in alg:
            calls[name]["algorithmic_GB"] = round(alg[name] / 1e9, 4)
            calls[name]["GBps"] = round(alg[name] / 1e6 / ms, 1)
            calls[name]["hbm_frac"] = round(alg[name] / 1e6 / ms / HBM_PEAK_GBS, 4)

    # matrix-unit view of the verify pass (what matters once a batch puts hundreds of rows through it):
    # algorithmic FLOPs = 2 x target parameters x verified rows, against the dense f16 MFMA peak
    if "verify" in calls:
        rows = nb * (main_run["mean_gamma"] + 1.0)
        flops = weight_bytes(w["target"], L) * rows          # 2 FLOPs per weight per row = bytes x rows for 2-byte weights
        tf = flops / 1e9 / calls["verify"]["mean_ms"]
        calls["verify"].update({"rows": round(rows, 1), "algorithmic_TFLOP": round(flops / 1e12, 4), "TFLOPs": round(tf, 1),
                                "mfma_frac": round(tf / MFMA_PEAK_TFLOPS, 4)})

    context = {}
    if not a.no_context:
        n_ctx = max(8, K // 4)
        fresh(); run_steps(sess, 3, mode, 3, batch, fixed_gamma=0)
        context["autoregressive_tok_s"] = round(run_steps(sess, n_ctx, mode, 3, batch, fixed_gamma=0)["tok_s"], 2)
        for g in (4, 8):
            fresh(); run_steps(sess, 3, mode, 3, batch, fixed_gamma=g)
            context[f"fixed_gamma_{g}_tok_s"] = round(run_steps(sess, n_ctx, mode, 3, batch, fixed_gamma=g)["tok_s"], 2)

    cpu = None
    if host is not None:
        cpu = cpu_baseline(w, host[0], host[1], host[2], prompt, 1 if mode == B.SAMPLE else 0)
        if a.cpu_one_thread:
            one = cpu_baseline(w, host[0], host[1], host[2], prompt, 1 if mode == B.SAMPLE else 0, threads=1)
            cpu["one_thread"] = {"value": one["value"], "cores": one["cores"], "sample": one["sample"]}
    ceiling = stream_ceiling(torch, B, w["target"] if w["dtype"] == "bf16" else None, L)

    if a.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # HBM bytes per launch counted by rocprofv3 (FETCH_SIZE / WRITE_SIZE, scaled by a plain copy):
    # taken from the committed summary of the same workload, if there is one
    traffic = None
    tf = os.path.join(ROOT, "profiles", f"gemm_w16_{a.workload}_hbm_traffic.txt")
    if os.path.exists(tf) and a.layers is None:
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = float(line.split("=", 1)[1])

    achieved = gemm_bytes / 1e9 / (gemm_ms / 1e3) if gemm_ms > 0 else 0.0
    # the same bytes at the rate of a kernel that only reads them, one cold launch per matrix (see stream_ceiling)
    floor_gbps = None
    fl = ceiling.get("per_launch_read_floor")
    if fl:
        floor_gbps = weight_bytes(w["target"], L) / 1e9 / (fl["pass_ms_without_attention"] / 1e3)
    out = {
        "metric": "decode tokens/s (7B-shape target, bs1) + verify-step achieved HBM GB/s",
        "value": round(main_run["tok_s"], 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(main_run["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f16 MFMA, f32 accumulate (bf16 weights held as f16; target activations as f16 hi + lo parts; f16 KV cache)"
                  if w["dtype"] == "bf16" else "f32"),
        "data": "synthetic",
        "config": {"workload": f"{a.workload}: {L}-layer d{w['target']['d_model']} target + {w['draft']['n_layers']}-layer "
                               f"d{w['draft']['d_model']} draft, prompt {n_prompt if nb == 1 else lens}, "
                               f"{'sampling T=1' if mode else 'greedy'}, gamma_max {w['gamma_max']}, "
                               f"b {w['block']}, beta {round(w['beta'], 3) if nb == 1 else 'U[1,5] per sequence'}, t0 {w['t0']}, rho {w['rho']}",
                   "batch": nb, "new_tokens": main_run["tokens"]},
        "tau": round(main_run["tau"], 3), "mean_gamma": round(main_run["mean_gamma"], 3),
        # realised acceptance rate by draft position (accepted / tested at that position), to set beside the
        # acceptance-versus-position figure of Sec. 3.1; positions never reached are null
        "acceptance_by_position": [round(a / r, 3) if r else None
                                   for a, r in zip(main_run["accepted"][:w["gamma_max"]], main_run["reached"][:w["gamma_max"]])],
        "tested_by_position": main_run["reached"][:w["gamma_max"]],
        "stream_ceiling": ceiling,
        "forwards": counts, "verify_GBps": calls.get("verify", {}).get("GBps"),
        "calls": calls, "context": context,
        "prefill": {"ms": round(prefill_ms, 2), "tokens": int(sum(lens)), "tok_s": round(sum(lens) / prefill_ms * 1e3, 1)},
        "roofline": {"bound": "hbm", "kernel": ("gemm_w16_kernel" if nb == 1 else "gemm_wide_kernel / gemm_w16_kernel")
                               + ", target-model launches (template TAG 0), all shapes",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "frac_of_streaming_read": round(achieved / ceiling["streaming_read_GBps"], 4),
                     "read_floor_GBps": round(floor_gbps, 1) if floor_gbps else None,
                     "frac_of_read_floor": round(achieved / floor_gbps, 4) if floor_gbps else None,
                     "launches": int(n_launch), "avg_launch_us": round(1e3 * gemm_ms / max(1, n_launch), 3),
                     "avg_launch_bytes": round(gemm_bytes / max(1, n_launch), 1)},
        "cpu_baseline": cpu,
    }
    sess.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
