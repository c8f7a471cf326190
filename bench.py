"""Throughput of the verification step on one MI355X, with roofline figures and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu]

A "step" is one ot_verify_step over one synthetic batch: LM-head projection with the target rows' softmax partials,
and in the same launch the draft softmax statistics and the translation (direct map + n-gram cache); then acceptance,
residual masses and the final-token draw.
The workload is the configuration the headline metric is quoted on: Llama3-8B-shaped target, V_t = 128256,
B = 16 sequences x k = 8 drafted tokens, bf16 (configuration 4).  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def lm_head_bytes(M, d, V_t):
    """Algorithmic HBM bytes of one LM-head launch: W read once, H read once, fp32 logits written once."""
    return 2 * d * V_t + 2 * M * d + 4 * M * V_t


def kernel_sources_digest():
    """Digest of the kernel sources: a counter measurement is valid for exactly the code it was taken on."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2507_02659_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp")):
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def read_traffic_note(path):
    """HBM bytes per LM-head launch measured with rocprofv3 --pmc (two runs: FETCH_SIZE, WRITE_SIZE), from the
    committed summary -- but only if that summary was taken on the kernel sources of this tree; otherwise None."""
    value, stamp = None, None
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("hbm_bytes_per_launch:"):
                    value = float(line.split(":")[1].split()[0])
                elif line.startswith("kernel_sources_sha:"):
                    stamp = line.split(":")[1].strip()
    except OSError:
        return None
    return value if stamp == kernel_sources_digest() else None


def measure_cliffs(torch, Verifier):
    """Step time at the capacity edges the header documents: B = 255 / 256 (fused launch against separate passes) at a
    mid-size bf16 head, and the one-thread-per-logit fp32 head."""
    from workloads import CaseSpec, make_case
    out = {}
    for name, B, dtype in (("bf16_B255", 255, "bf16"), ("bf16_B256", 256, "bf16"), ("f32_B16", 16, "f32")):
        spec = CaseSpec(name=name, dtype=dtype, d=1024, V_t=32000, V_d=8000, k=[3] * B, temperature=[1.0] * B, n_direct=6000,
                        n_ngram=2000, ngram_len=(2, 4), plant_cover=0.3, data_seed=400 + B, philox_seed=1)
        case = make_case(spec)
        v = Verifier.for_case(case)
        inp = v.upload(case)
        for i in range(5):
            v.step(inp, step=i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = 30
        for i in range(n):
            v.step(inp, step=i)
        torch.cuda.synchronize()
        out[name] = {"B": B, "rows_M": case.M, "d": 1024, "V_t": 32000, "us_per_step": round(1e6 * (time.perf_counter() - t0) / n, 1)}
        v.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="BASELINE configuration 1..5 (default: the headline one)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--cliffs", action="store_true",
                    help="also time the capacity edges: 255 against 256 sequences (where the LM-head launch stops hosting "
                         "the statistics and the draft side) and the fp32 head at a mid size")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) so that a rocprofv3 --pmc run of this "
                         "command can scale FETCH_SIZE / WRITE_SIZE of the LM-head kernel against it")
    ap.add_argument("--cold-weights", type=int, default=1, metavar="N",
                    help="rotate the steps over N contexts, each with a private copy of the LM head, so that no step finds "
                         "its weights in the 256 MB last-level cache (matters where W is that small: configuration 2)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    from workloads import baseline_spec, make_case

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the verification path has no CPU fallback")

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    t0 = time.time()
    case = make_case(baseline_spec(args.config))
    sys.stderr.write(f"[bench] generated {case.name} in {time.time() - t0:.1f}s: B={case.B} M={case.M} K={case.K} "
                     f"d={case.d} V_t={case.V_t} V_d={case.V_d}\n")
    v = Verifier.for_case(case)
    inp = v.upload(case)
    from_logits = case.hidden is None
    # contexts the steps rotate over (one unless --cold-weights asks for more); all enqueue on the same stream
    ring = [(v, inp)]
    for _ in range(max(args.cold_weights, 1) - 1):
        vv = Verifier.for_case(case)
        ring.append((vv, vv.upload(case)))

    def run_step(i):
        vv, ii = ring[i % len(ring)]
        vv.step(ii, from_logits=from_logits, step=i)

    # per-kernel durations: HIP events recorded by the library on its own stream between the step's launches (each
    # event costs the stream about 5 us, so this pass is separate from the timed one)
    for vv, _ in ring:
        ot.ot_verify_profile(vv.ctx, True)
    # at least 200 steps: the averages should be those of a running service, and this chip takes some ten
    # milliseconds of load to settle its clocks (the first 50 steps of a process run about 10 % slower)
    n_prof = min(max(args.steps, 200), 1000)
    for i in range(n_prof):
        run_step(i)
    stage_us, n_read = {}, 0
    for vv, _ in ring:
        stage_ms, n = ot.ot_verify_profile_read(vv.ctx)
        ot.ot_verify_profile(vv.ctx, False)
        n_read += n
        for k, t in stage_ms.items():
            stage_us[k] = stage_us.get(k, 0.0) + 1e3 * t
    stage_us = {k: t / max(n_read, 1) for k, t in stage_us.items()}

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        run_step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = 1e3 * elapsed / args.steps
    value = case.K * args.steps / elapsed

    # one more step with the benchmark's own step index, kept for the parity note below
    v.step(inp, from_logits=from_logits, step=case.step)
    gpu = v.results(inp)

    M, K, d, V_t, V_d = case.M, case.K, case.d, case.V_t, case.V_d
    esz = 2 if case.dtype == "bf16" else 4
    gemm_bytes = lm_head_bytes(M, d, V_t) if esz == 2 else 4 * d * V_t + 4 * M * d + 4 * M * V_t
    gemm_s = stage_us["lm_head"] * 1e-6
    achieved = gemm_bytes / gemm_s / 1e9 if gemm_s > 0 else 0.0
    # what follows the LM head: with fused statistics one launch (merge of the partials + acceptance + draw), else
    # statistics, translation + acceptance, draw
    fused = esz == 2 and M > 16 and case.B <= 255 and not from_logits
    tail_us = ms_per_step * 1e3 - stage_us["lm_head"]
    extra = {
        "stage_us": {k: round(x, 2) for k, x in stage_us.items()},
        "stage_us_note": "HIP events on the library's stream; every event adds about 5 us to the stage after it",
        "after_lm_head_us": round(tail_us, 2),
        "lm_head_tflops": round(2.0 * M * d * V_t / gemm_s / 1e12, 1) if gemm_s > 0 else None,
        "lm_head_frac_mfma_peak": round(2.0 * M * d * V_t / gemm_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4) if gemm_s > 0 else None,
        "rows_per_s": round(M * args.steps / elapsed, 1),
        "step_hbm_bytes": gemm_bytes + esz * K * V_d + (16 * M * ((V_t + 255) // 256) if fused else 4 * M * V_t)
                          + case.B * (4 * V_t + esz * V_d + 4 * V_t),
    }
    if len(ring) > 1:
        extra["cold_weights"] = f"steps rotate over {len(ring)} contexts with private copies of the LM head"
    extra["row_statistics"] = "lm_head epilogue, draft side in the same launch" if fused else "separate pass over the logits"

    # The softmax pass on its own (the metric's "% HBM BW (softmax)"): the same batch through
    # ot_verify_step_from_logits with the logits the LM head just produced, so that the statistics kernel reads all
    # M target rows (fp32) and all K draft rows once.
    if not from_logits and K > 0:
        ws = v.workspace(M, K, with_logits=True)
        inp["target_logits"] = torch.from_numpy(np.ascontiguousarray(ws["logits"])).to("cuda")
        del ws
        ot.ot_verify_profile(v.ctx, True)
        for i in range(50):
            v.step(inp, from_logits=True, step=i)
        sm_ms, sm_n = ot.ot_verify_profile_read(v.ctx)
        ot.ot_verify_profile(v.ctx, False)
        sm_us = 1e3 * sm_ms["softmax_stats"] / max(sm_n, 1)
        sm_bytes = 4 * M * V_t + esz * K * V_d
        extra["softmax_pass"] = {"kernel": "softmax_stats_kernel", "us": round(sm_us, 2), "algorithmic_bytes": sm_bytes,
                                 "gbs": round(sm_bytes / (sm_us * 1e-6) / 1e9, 1),
                                 "frac_hbm_peak": round(sm_bytes / (sm_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                 "note": "event-timed like stage_us (includes about 5 us of event cost); the rocprofv3 figure is "
                                         "in profiles/kernel_stats_cfg4_softmax_pass.txt"}
        inp["target_logits"] = None
        v.step(inp, from_logits=False, step=case.step)       # back to the batch's own step for what follows

    # forward values of the hybrid distillation loss on the same batch (the pass that follows a step when the
    # drafter is trained online): reverse KL on every direct-mapping token, NLL on n-gram tokens
    if K > 0:
        n_loss = 50
        v.distill_loss(inp, from_logits=from_logits)
        torch.cuda.synchronize()
        t_l = time.perf_counter()
        for _ in range(n_loss):
            loss = v.distill_loss(inp, from_logits=from_logits, sync=False)
        v.synchronize()
        loss_us = 1e6 * (time.perf_counter() - t_l) / n_loss
        loss = v.distill_loss(inp, from_logits=from_logits)
        kl_rows = int(loss["n_dm"])
        loss_bytes = kl_rows * (4 * V_t + 4 * V_t + esz * int((case.direct_map >= 0).sum()))   # logit row, inverse map, gathered draft row
        extra["distill_loss"] = {"us_per_call": round(loss_us, 2), "kl_rows": kl_rows, "algorithmic_bytes": loss_bytes,
                                 "gbs": round(loss_bytes / (loss_us * 1e-6) / 1e9, 1), "loss": round(loss["loss"], 6)}
    extra["step_frac_hbm_roofline"] = round(extra["step_hbm_bytes"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if args.cliffs:
        extra["cliffs"] = measure_cliffs(torch, Verifier)

    result = {
        "metric": "verified draft positions/sec at V_t=128k",
        "value": round(value, 1),
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": case.dtype,
        "data": "synthetic",
        "config": {"workload": f"BASELINE configuration {args.config}: {case.name}", "B": case.B, "k": int(case.k.max()),
                   "rows_M": M, "draft_positions_K": K, "d": d, "V_t": V_t, "V_d": V_d,
                   "ngram_entries": int(case.ngram_target_ids.size)},
        "roofline": {
            "kernel": "lmhead_bf16_wide_kernel" if esz == 2 else "lmhead_f32_kernel",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": gemm_bytes,
            "avg_launch_us": round(stage_us["lm_head"], 2),
            "traffic": read_traffic_note(os.path.join(ROOT, "profiles", f"lm_head_cfg{args.config}_hbm_traffic.txt")),
        },
        "extra": extra,
    }

    if not args.no_cpu:
        from oracle import verify as ov
        import parity
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        t1 = time.perf_counter()
        ref = ov.verify_case(case)
        reps = 1
        while time.perf_counter() - t1 < 12.0 and reps < 64:      # bounded sample: about 10-20 s of CPU work
            case.step = 1000 + reps
            ov.verify_case(case)
            reps += 1
        case.step = baseline_spec(args.config).step
        cpu_s = time.perf_counter() - t1
        result["cpu_baseline"] = {
            "value": round(reps * case.K / cpu_s, 2), "unit": "positions/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{reps} whole steps of the same workload ({case.B} sequences, {case.K} drafted positions each, "
                      f"different Philox steps), NumPy float64, {cpu_s:.1f}s",
        }
        rep = parity.compare(case, gpu, ref, logits_from_gpu=not from_logits)
        result["parity"] = {"summary": rep.summary(), "failures": len(rep.failures)}
    for vv, _ in ring:
        vv.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
