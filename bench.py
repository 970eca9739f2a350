#!/usr/bin/env python3
"""Benchmark of the adaptive self-speculative decoding engine on one MI355X.

One timed step = one greedy decode of the workload's new tokens after its prompt has been
processed (the prompt pass runs once, untimed: the hot path is the draft / verify loop; the
prompt's KV cache and all weights are resident in HBM when the timed region starts).
`value` is plain greedy decoding (draft length 0: every token is one single-row pass of the
verification kernels), the figure the HBM-roofline target is stated for; the speculative
runs (ADMG mask from the prompt's ACS, and the all-keep bracket) are reported beside it with
their acceptance, which on random-init weights is an artefact of the init.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E peak


def cpu_baseline(shape, seed, n_prompt=2, n_decode=6):
    """The oracle as it stands, timed on this host: a short prompt plus a few greedy tokens."""
    import asd_inputs as si
    import oracle
    t0 = time.time()
    orc = oracle.Oracle(shape, n_prompt + n_decode + 1, kv_storage=True)
    for t, l, a in si.all_tensors(shape, seed):
        orc.set_weight(t, l, a)
    t_load = time.time() - t0
    prompt = si.prompt(seed, n_prompt, shape.vocab)
    t0 = time.time()
    orc.forward(prompt, 0, want_logits=False)
    t_prompt = time.time() - t0
    tok = np.array([1], np.int32)
    t0 = time.time()
    for i in range(n_decode):
        r = orc.forward(tok, n_prompt + i, want_logits=False)
        tok = r["argmax"][:1].copy()
    t_dec = time.time() - t0
    orc.close()
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n_decode / t_dec, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{shape.name} shape, full depth and width: {n_prompt}-token prompt then {n_decode} plain greedy "
                      f"tokens (decode phase timed: {t_dec:.1f} s; prompt {t_prompt:.1f} s; weight generation "
                      f"{t_load:.1f} s not counted)"}


def read_traffic(path):
    """HBM bytes per launch of the dominant kernel from the committed counter summary, or None."""
    try:
        for ln in open(path):
            if ln.startswith("TRAFFIC_BYTES_PER_LAUNCH"):
                return float(ln.split("=")[1])
    except OSError:
        pass
    return None


def progress(msg):
    """One line on stderr per finished phase: long workloads stay visibly alive; stdout carries only the JSON line."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def copy_rate(eng):
    """GB/s of a plain copy kernel (192 MiB read + 192 MiB written); None when the engine's scratch region is too small
    for that (the tiny workload), where the figure would not be an HBM number anyway."""
    import paper_2410_01028_amd as asd
    try:
        ms = eng.copy_bench(192 << 20, 10)
    except asd.AsdError:
        return None
    return round(2 * (192 << 20) / ms / 1e6, 1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="7b", help="tiny | 7b | 13b | 7b-long | 70b")
    ap.add_argument("--draft-len", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the speculative / per-pass extras")
    ap.add_argument("--n-new", type=int, default=None, help="override the workload's number of new tokens (profiling runs)")
    ap.add_argument("--copy-only-extra", action="store_true", help="with --no-extras: still run the plain copy kernel (counter calibration)")
    ap.add_argument("--only-verify-passes", type=int, default=0, metavar="N",
                    help="counter runs: after the prompt pass launch N eager (draft_len+1)-row verification passes and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    import asd_inputs as si
    import paper_2410_01028_amd as asd

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    shape = si.SHAPES[args.workload]
    seed = 0
    k = args.draft_len if args.draft_len is not None else shape.draft_len
    P, N = shape.prompt_len, (args.n_new or shape.n_new)
    max_seq = P + N + 16
    eng = asd.Engine(asd.make_config(shape, max_seq, page_tokens=256))
    eng.init_synthetic(seed)
    prompt = si.prompt(seed, P, shape.vocab)
    L2 = 2 * shape.n_layers

    progress(f"{shape.name}: weights ready")
    first, acs, _ = eng.prefill(prompt)          # untimed: first touch of every weight, lazy runtime set-up
    torch.cuda.synchronize()
    progress("first prompt pass done")
    if args.only_verify_passes:
        ms, by = eng.time_pass(k + 1, None, args.only_verify_passes, False)
        print(json.dumps({"verify_rows": k + 1, "ms_per_pass": round(ms, 4), "GBps": round(by / ms / 1e6, 1)}), flush=True)
        return
    pf_prof = eng.profile_prefill(prompt) if (P > 16 and not args.no_extras) else None     # resets the cache: before the timed passes
    t0 = time.time()
    for _ in range(3):
        first, acs, _ = eng.prefill(prompt)
    torch.cuda.synchronize()
    t_prefill = (time.time() - t0) / 3

    def decode_step(draft_len, **kw):
        eng.truncate(P)
        return eng.decode(first, N - 1, draft_len, **kw)

    progress(f"prompt pass timed: {t_prefill * 1e3:.1f} ms")
    for _ in range(args.warmup):
        decode_step(0)
        progress("warm-up decode done")
    torch.cuda.synchronize()
    t0 = time.time()
    for i in range(args.steps):
        plain, st_plain, _ = decode_step(0)
        progress(f"timed decode {i + 1}/{args.steps} done")
    torch.cuda.synchronize()
    total = time.time() - t0
    ms_per_step = total / args.steps * 1e3
    value = (N - 1) * args.steps / total

    out = {
        "metric": "greedy decode tokens/s at batch 1", "value": round(value, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype else "f32",
        "data": "synthetic (seeded random-init weights, uniform-random prompt; stands in for Llama-2 checkpoints and "
                "CNN/DM, XSum, HumanEval prompts)",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers, d_model {shape.d_model}, {shape.n_heads} heads "
                               f"({shape.n_kv_heads} KV) x {shape.head_dim}, FFN {shape.d_ffn}, vocab {shape.vocab}; "
                               f"batch 1, prompt {P}, {N} greedy tokens",
                   "mode": "plain greedy (draft length 0), decode phase after the prompt pass", "draft_len_spec": k},
        "prefill_ms": round(t_prefill * 1e3, 2),
        "e2e_tokens_per_s": round(N / (t_prefill + ms_per_step / 1e3), 2),
    }
    # the prompt pass is the one matrix-core-bound step: flops of the weight contractions (each counted once, although
    # bf16 activations go through the matrix cores as two planes) plus causal attention, against the dense bf16 peak
    qd, kvd = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    w_flop = 2.0 * P * shape.n_layers * (shape.d_model * (qd + 2 * kvd) + qd * shape.d_model + 3 * shape.d_model * shape.d_ffn)
    a_flop = 2.0 * 2.0 * shape.n_layers * qd * P * (P + 1) / 2
    out["prefill"] = {"ms": round(t_prefill * 1e3, 2), "prompt_tokens_per_s": round(P / t_prefill, 1),
                      "model_TFLOPs": round((w_flop + a_flop) / t_prefill / 1e12, 1),
                      "frac_of_bf16_mfma_peak": round((w_flop + a_flop) / t_prefill / 2.5e15, 4),
                      "matrix_core_planes": 2 if shape.dtype else 1}
    if pf_prof:
        # event pair around every launch of one prompt pass; flops of a class = its contractions, each multiply-add once
        out["prefill"]["kernels"] = {n: {"avg_us": round(v["ms"] / v["launches"] * 1e3, 1), "launches": v["launches"],
                                         "TFLOPs": round(v["flops"] / v["ms"] / 1e9, 1) if v["flops"] else None}
                                     for n, v in pf_prof.items() if n != "ms_total" and v["launches"]}
        gu = pf_prof["gateup"]
        tf = gu["flops"] / gu["ms"] / 1e9
        planes = 2 if shape.dtype else 1
        out["prefill"]["roofline"] = {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0 if shape.dtype else 157.3, "unit": "TFLOP/s",
                                      "frac": round(tf / (2500.0 if shape.dtype else 157.3), 4),
                                      "kernel": "pf_gemm_kernel<PF_GU> (prompt-block gate/up projection + SiLU*mul)",
                                      "flops_per_launch": gu["flops"] / gu["launches"], "avg_launch_us": round(gu["ms"] / gu["launches"] * 1e3, 2),
                                      "matrix_core_issue_frac": round(tf * planes / (2500.0 if shape.dtype else 157.3), 4)}

    # ---- roofline of the dominant kernel (gate/up projection GEMM), HIP events on the engine's stream
    reps = 5
    acc = {}
    for _ in range(reps):
        pf = eng.profile_forward(1)
        for name, v in pf.items():
            if name == "ms_total":
                continue
            a = acc.setdefault(name, {"ms": 0.0, "launches": 0, "bytes": 0.0})
            a["ms"] += v["ms"]; a["launches"] += v["launches"]; a["bytes"] += v["bytes"]
    # dominant kernel: the gate/up GEMM launched back to back over the layers' (distinct) weights, one event pair
    eng.truncate(P)
    gu_us, bytes_per_launch = eng.time_step_class("gateup", 1, 10)
    achieved = bytes_per_launch / gu_us / 1e3
    out["roofline"] = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(achieved / HBM_PEAK_GBS, 4),
                       "traffic": read_traffic(os.path.join(ROOT, "profiles", f"gemm_gateup_{shape.name}_hbm_traffic.txt")),
                       "kernel": f"gemm_kernel<{'BF16' if shape.dtype else 'F32'}, EPI_GU> (gate/up projection + SiLU*mul)",
                       "bytes_per_launch": bytes_per_launch, "avg_launch_us": round(gu_us, 2)}
    # every class inside a pass, an event pair around each launch (includes the event overhead of ~2 us)
    out["kernels"] = {n: {"avg_us": round(v["ms"] / v["launches"] * 1e3, 2),
                          "GBps": round(v["bytes"] / max(v["ms"], 1e-12) / 1e6, 1) if v["bytes"] else None}
                      for n, v in acc.items() if v["launches"]}

    if args.no_extras and args.copy_only_extra:
        out["copy_kernel_GBps"] = copy_rate(eng)
    if not args.no_extras:
        eng.truncate(P)
        ms1, by1 = eng.time_pass(1, None, 30, True)
        msv, byv = eng.time_pass(k + 1, None, 30, True)
        mask = asd.admg(acs[0::2], 0.985, 3, 2)
        msd, byd = eng.time_pass(1, mask, 30, True)
        out["passes"] = {
            "full_1row": {"ms": round(ms1, 4), "GBps": round(by1 / ms1 / 1e6, 1), "frac_peak": round(by1 / ms1 / 1e6 / HBM_PEAK_GBS, 4)},
            f"verify_{k + 1}rows": {"ms": round(msv, 4), "GBps": round(byv / msv / 1e6, 1), "frac_peak": round(byv / msv / 1e6 / HBM_PEAK_GBS, 4)},
            "draft_admg_1row": {"ms": round(msd, 4), "GBps": round(byd / msd / 1e6, 1), "frac_peak": round(byd / msd / 1e6 / HBM_PEAK_GBS, 4),
                                "kept_attn": int(shape.n_layers - mask[0::2].sum()), "kept_mlp": int(shape.n_layers - mask[1::2].sum())},
        }
        out["copy_kernel_GBps"] = copy_rate(eng)
        progress("per-pass timings done")
        spec = {}
        # Table 2's setting for Llama-2-7B; a cosine-only setting (no periodic rule) with the threshold moved to where
        # this random-init model's ACS values lie; and the all-keep bracket (every draft accepted, no layer skipped)
        for name, kw in (("admg_a0.985_m3_n2", dict(alpha=0.985, m=3, n=2)),
                         ("admg_a0.9999_m0_n0", dict(alpha=0.9999, m=0, n=0)),
                         ("all_keep", dict(fixed_mask=np.zeros(L2, np.uint8))),
                         # loop extensions on the cosine-only setting: running-ACS mask refresh; adaptive draft exit with
                         # at most 6 drafts and a threshold at this model's (tiny, random-init) draft confidences
                         ("admg_a0.9999_m0_n0_refresh", dict(alpha=0.9999, m=0, n=0, refresh=True)),
                         ("admg_a0.9999_m0_n0_adaptive_exit_kmax6", dict(alpha=0.9999, m=0, n=0, exit_mode=1, gamma0=0.003, ar0=1.0,
                                                                        ar_target=0.9, eps=0.0005, beta1=0.5, beta2=0.9, kmax=6))):
            kw = dict(kw)
            kk = kw.pop("kmax", k)
            decode_step(kk, **kw)
            torch.cuda.synchronize()
            progress(f"speculative {name}: warm-up done")
            t0 = time.time()
            toks, st, used = decode_step(kk, **kw)
            dt = time.time() - t0
            spec[name] = {"tokens_per_s": round((N - 1) / dt, 2), "speedup_vs_plain": round((N - 1) / dt / value, 3),
                          "cycles": st["cycles"], "drafted": st["drafted"], "accepted": st["accepted"],
                          "removed_attn": int(used[0::2].sum()), "removed_mlp": int(used[1::2].sum()), "mask_changes": st["mask_changes"],
                          "tokens_equal_plain": bool(np.array_equal(toks, plain))}
            progress(f"speculative {name}: {spec[name]['tokens_per_s']} tokens/s")
        out["speculative"] = spec
        # sampled decoding at the paper's higher temperature: plain sampling of the full model against speculative sampling
        samp = {}
        for name, kk, kw in (("plain_T0.6", 0, dict(fixed_mask=np.zeros(L2, np.uint8))),
                             ("admg_a0.9999_m0_n0_T0.6", k, dict(alpha=0.9999, m=0, n=0))):
            kw = dict(kw, temperature=0.6, seed=1, sample_index0=1)
            decode_step(kk, **kw)
            torch.cuda.synchronize()
            t0 = time.time()
            toks, st, used = decode_step(kk, **kw)
            dt = time.time() - t0
            samp[name] = {"tokens_per_s": round((N - 1) / dt, 2), "cycles": st["cycles"], "drafted": st["drafted"],
                          "accepted": st["accepted"], "removed_attn": int(used[0::2].sum())}
            progress(f"sampled {name}: {samp[name]['tokens_per_s']} tokens/s")
        samp["speedup"] = round(samp["admg_a0.9999_m0_n0_T0.6"]["tokens_per_s"] / samp["plain_T0.6"]["tokens_per_s"], 3)
        out["sampled"] = samp

    eng.close()
    del eng
    torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        progress("GPU part done; timing the CPU oracle")
        if shape.name == "tiny":
            out["cpu_baseline"] = cpu_baseline(shape, seed, 8, 24)
        else:
            # about ten seconds of decoding on the box's 16 host threads: 40 tokens at the 7B size, fewer for larger models
            per_tok = shape.n_layers * (shape.d_model * (shape.q_dim + 2 * shape.kv_dim) + shape.q_dim * shape.d_model
                                        + 3 * shape.d_model * shape.d_ffn) + shape.vocab * shape.d_model
            out["cpu_baseline"] = cpu_baseline(shape, seed, 2, max(4, int(40 * 6.6e9 / per_tok)))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
