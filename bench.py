#!/usr/bin/env python3
"""Benchmark of the autoregressive AED decoder path on one MI355X.

A step = one pass of the whole path over one batch of seeded synthetic input:
cross-attention K/V precompute for all layers, then greedy decoding of the
4-token prompt plus max_new tokens through the captured launch graph.  Inputs
(weights, encoder states, prompts) are resident in HBM before the timed region.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None when there is none for
    this kernel and workload or the kernel's source has changed since the counters were taken."""
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json"))).get(kernel)
        if not rec or rec["workload"] != workload:
            return None
        h = hashlib.sha256(open(os.path.join(ROOT, rec["source"]), "rb").read()).hexdigest()[:16]
        return rec["traffic_bytes_per_launch"] if h == rec["sha256_16"] else None
    except (OSError, ValueError, KeyError):
        return None


def run_workload(name, steps, warmup, want_roofline, eager=False, no_prefill=False, kv_fp8=False):
    import numpy as np
    import torch
    from paper_2503_05931_amd import binding, workloads as W

    wl = W.make(name)
    cfg = wl.cfg
    cfg.kv_fp8 = 1 if kv_fp8 else 0  # optional 8-bit (E4M3) key / value caches; the default run keeps them in bf16
    B = cfg.batch
    # eager: the library is given the default (NULL) stream, on which it launches every kernel directly
    # instead of replaying a captured graph (used for hardware-counter runs)
    # the prompt positions before the last go through the layers in one pass (rows: 16-aligned batch per position)
    prefill_rows = 0 if no_prefill else min(cfg.prompt_len - 1, 8) * ((B + 15) // 16 * 16)
    dec = binding.Decoder(cfg, wl.weights, max_batch=B, max_total_enc_frames=int(wl.enc_lens.sum()),
                          max_dec_len=cfg.max_dec_len, prefill_rows=prefill_rows,
                          stream=torch.cuda.default_stream(torch.device("cuda:0")) if eager else None)
    enc = dec.to_device(wl.enc)
    prompt = torch.from_numpy(wl.prompt).to(dec.device)
    out_tokens = torch.empty((B, cfg.max_new), dtype=torch.int32, device=dec.device)
    out_lens = torch.empty(B, dtype=torch.int32, device=dec.device)
    mnps = wl.max_new_per_seq
    torch.cuda.synchronize()

    def one_step():
        dec.aed_cross_kv_precompute(enc, wl.enc_lens)
        dec.aed_greedy_decode(prompt, cfg.max_new, max_new_per_seq=mnps, out_tokens=out_tokens, out_lens=out_lens)

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tokens = int(out_lens.sum().item())
    res = {
        "workload": name,
        "tokens_per_step": tokens,
        "ms_per_step": 1e3 * dt / steps,
        "tokens_per_s": tokens * steps / dt,
    }
    # decode alone (cross K/V already resident), and the precompute alone
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dec.aed_cross_kv_precompute(enc, wl.enc_lens)
    torch.cuda.synchronize()
    res["precompute_ms"] = 1e3 * (time.perf_counter() - t0)
    t0 = time.perf_counter()
    dec.aed_greedy_decode(prompt, cfg.max_new, max_new_per_seq=mnps, out_tokens=out_tokens, out_lens=out_lens)
    torch.cuda.synchronize()
    d2 = time.perf_counter() - t0
    res["decode_only_tokens_per_s"] = tokens / d2
    # decoder steps of the loop: without prefill the prompt positions before the last are steps too
    res["decode_ms_per_token_step"] = 1e3 * d2 / ((cfg.prompt_len - 1 if no_prefill else 0) + cfg.max_new)
    if wl.durations_s is not None:
        res["decoder_rtfx"] = float(np.sum(wl.durations_s)) * steps / dt

    if want_roofline:
        # Per-kernel-class time at the middle of the decode: run half of the steps, then replay each
        # class over all layers between HIP events on the decoder's stream.
        dec.aed_cross_kv_precompute(enc, wl.enc_lens)
        half = max(1, cfg.max_new // 2)
        dec.aed_greedy_decode(prompt, half)
        classes = [binding.K_LN_QKV, binding.K_SELF_ATTN, binding.K_SELF_OUT, binding.K_LN_CROSSQ,
                   binding.K_CROSS_ATTN, binding.K_CROSS_OUT, binding.K_LN_FFN1, binding.K_FFN2, binding.K_CROSS_KV]
        per = {}
        for k in classes:
            dec.aed_time_kernels(k, 2)  # warm
            ms, n = dec.aed_time_kernels(k, 20)
            if n == 0:
                continue   # this class is part of another class's launch at this batch size
            nbytes, flops = dec.aed_kernel_work(k)
            per[binding.KERNEL_NAMES[k]] = {"us": 1e3 * ms / n, "bytes": nbytes, "flops": flops,
                                            "GBps": nbytes / (ms / n * 1e-3) / 1e9,
                                            "TFLOPs": flops / (ms / n * 1e-3) / 1e12}
        # the once-per-batch cross K/V GEMM is MFMA-bound: reported on its own, not as the step's dominant kernel
        ckv = per.pop("cross_kv")
        res["mfma"] = {"kernel": "cross_kv", "bound": "mfma", "achieved": ckv["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                       "unit": "TFLOP/s", "frac": ckv["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, "avg_launch_us": ckv["us"],
                       "flops_per_launch": ckv["flops"]}
        dom = max(per, key=lambda k: per[k]["us"])
        p = per[dom]
        res["kernels"] = {k: {"us": round(v["us"], 2), "GBps": round(v["GBps"], 1)} for k, v in per.items()}
        # the projection products as MFMA work (flops / time against the dense bf16 peak); meaningful from batch 256 on,
        # below that they are weight streams
        res["mfma_projection"] = {
            "M": B, "bound": "mfma", "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "kernels": {k: {"us": round(per[k]["us"], 2), "achieved": round(per[k]["TFLOPs"], 1),
                            "frac": round(per[k]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)}
                        for k in ("ln_qkv", "ln_ffn1", "ffn2") if k in per}}
        att = {k: per[k] for k in ("self_attn", "cross_attn")}
        res["attention_hbm"] = {k: {"us": round(v["us"], 2), "achieved": round(v["GBps"], 1),
                                    "frac": round(v["GBps"] / HBM_PEAK_GBS, 4), "bytes_per_launch": v["bytes"]}
                                for k, v in att.items()}
        res["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": p["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": p["GBps"] / HBM_PEAK_GBS, "traffic": None if kv_fp8 else measured_traffic(dom, name),
                           "avg_launch_us": p["us"], "algorithmic_bytes_per_launch": p["bytes"]}
    dec.close()
    return res, wl


def run_ragged(steps, warmup):
    """Ragged-vs-padded stress on the 24-layer decoder, batch 128: the same 2048 samples (a) in random batches,
    (b) 2D-bucketed into cells of similar (encoder length, output length), (c) as (a) with every encoder
    length raised to the batch maximum and no forced end, which is what a padded tensor costs, and (d) as one
    request queue through 128 slots with slot refill.  Forced EOS at
    each sample's target length; tokens counted are the real (unpadded) ones."""
    import numpy as np
    import torch
    from paper_2503_05931_amd import binding, workloads as W

    wl = W.make("ragged24_b128", with_enc=False)
    cfg = wl.cfg
    pe, pd, perm = wl.extra["pool_enc"], wl.extra["pool_dec"], wl.extra["perm"]
    B = cfg.batch
    rng = np.random.default_rng(33)
    dec = binding.Decoder(cfg, wl.weights, max_batch=B, max_total_enc_frames=B * 500, max_dec_len=cfg.max_dec_len)
    prompts = torch.from_numpy(W.draw_prompts(cfg, rng, batch=2048)).to(dec.device)
    # encoder states: one [500, d] block per sample would be 2 GB; the values do not matter for timing, so every
    # sample reads its frames from one shared N(0,1) buffer
    frames = dec.to_device(W.bf16_round(rng.standard_normal((B * 500, cfg.d_model), dtype=np.float32)))
    out_tokens = torch.empty((B, cfg.max_new), dtype=torch.int32, device=dec.device)
    out_lens = torch.empty(B, dtype=torch.int32, device=dec.device)

    def run_case(batches, padded):
        tokens = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for idx in batches:
            lens = pe[idx]
            if padded:
                lens = np.full_like(lens, lens.max())
            total = int(lens.sum())
            dec.aed_cross_kv_precompute(frames[:total], lens)
            tgt = pd[idx]
            if padded:
                tgt = np.full_like(tgt, tgt.max())
            dec.aed_greedy_decode(prompts[torch.from_numpy(idx).to(dec.device)], int(cfg.max_new), max_new_per_seq=tgt,
                                  out_tokens=out_tokens, out_lens=out_lens)
            tokens += int(np.minimum(pd[idx], out_lens.cpu().numpy()).sum())
        torch.cuda.synchronize()
        return tokens, time.perf_counter() - t0

    # case (b): the library's 2D batch former, 8 duration bins x 2 output-length sub-bins, batches of B
    from paper_2503_05931_amd import batching
    former = batching.Bucketing(pe, pd, 8, 2)
    batch_of, bucket_of_batch = former.aed_bucketing_form_batches(pe, pd, batching.FLEXIBLE, np.full(16, B, np.int32))
    bucketed = [np.where(batch_of == t)[0] for t in range(len(bucket_of_batch))]
    n_formed = len(bucketed)
    bucketed = [x for x in bucketed if len(x) == B]   # timed: full batches only (the partial ones are counted below)
    dropped = {"partial_batches": n_formed - len(bucketed),
               "samples": int(len(pe) - sum(len(x) for x in bucketed))}
    cases = {"ragged_random": (W.random_batches(pe, pd, perm, B), False),
             "bucketed_2d": (bucketed, False),
             "padded_random": (W.random_batches(pe, pd, perm, B), True)}
    out = {}
    for name, (batches, padded) in cases.items():
        batches = batches[:max(1, steps)] if steps < len(batches) else batches
        if warmup:
            run_case(batches[:1], padded)
        tokens, dt = run_case(batches, padded)
        out[name] = {"tokens_per_s": tokens / dt, "batches": len(batches), "tokens": tokens, "seconds": dt,
                     "padding_enc": W.padding_fraction([pe[i] for i in batches]),
                     "padding_dec": W.padding_fraction([pd[i] for i in batches])}
    out["bucketed_2d"]["not_timed"] = dropped
    # case (d): the same samples as (a), in the same order, as one queue through B slots that are refilled as
    # sequences end.  The queue call takes every request's encoder states at once (values do not matter for timing).
    batches = cases["ragged_random"][0]
    batches = batches[:max(1, steps)] if steps < len(batches) else batches
    order = np.concatenate(batches)
    q_lens, q_tgt = pe[order], pd[order]
    torch.manual_seed(33)
    q_enc = torch.randn((int(q_lens.sum()), cfg.d_model), device=dec.device, dtype=torch.float32).to(torch.bfloat16)
    q_prompts = prompts[torch.from_numpy(order).to(dec.device)].contiguous()
    if warmup:
        n0 = len(batches[0])
        dec.aed_greedy_decode_queue(q_enc[:int(q_lens[:n0].sum())], q_lens[:n0], q_prompts[:n0], int(cfg.max_new),
                                    max_new_per_req=q_tgt[:n0])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _, lens_q, n_steps = dec.aed_greedy_decode_queue(q_enc, q_lens, q_prompts, int(cfg.max_new), max_new_per_req=q_tgt)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tokens = int(np.minimum(q_tgt, lens_q.cpu().numpy()).sum())
    out["ragged_queue"] = {"tokens_per_s": tokens / dt, "requests": int(len(order)), "slots": int(B), "tokens": tokens,
                           "seconds": dt, "decoder_steps": n_steps}
    dec.close()
    return out, cfg


def cpu_baseline(wl, n_seq=16, n_new=96):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import aed_oracle as O
    sub = wl.subset(list(range(min(n_seq, len(wl.enc_lens)))))
    m = O.Model(wl.cfg, wl.weights)
    t0 = time.perf_counter()
    m.greedy_decode(sub.enc, sub.enc_lens, sub.prompt, n_new)
    dt = time.perf_counter() - t0
    B = len(sub.enc_lens)
    return {"value": B * n_new / dt, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"first {B} sequences of the workload, cross K/V precompute + {wl.cfg.prompt_len}-token prompt "
                      f"+ {n_new} greedy tokens each ({dt:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="canary24_b64")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the extra workloads (4-layer decoder, large batch)")
    ap.add_argument("--no-large", action="store_true", help="skip the large-batch workload of the extra lines")
    ap.add_argument("--no-prefill", action="store_true",
                    help="feed the prompt one position per decoder step instead of prefilling it in one pass")
    ap.add_argument("--kv-fp8", action="store_true",
                    help="keep the attention keys / values as 8-bit E4M3 codes (an optional mode: its numbers are "
                         "not the bf16 headline figure)")
    ap.add_argument("--eager", action="store_true",
                    help="launch kernels directly on the default stream instead of replaying the captured graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known size to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters with)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the decoder shards by sequence with no exchange between GPUs, "
              "and this build runs on a single MI355X; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback)", file=sys.stderr)
        sys.exit(1)

    if args.workload == "ragged24_b128":
        cases, cfg = run_ragged(args.steps if args.steps != 5 else 16, args.warmup)
        a = cases["ragged_random"]
        print(json.dumps({
            "metric": "decoded tokens/sec at 1 MI355X (24L and 4L decoder) + % HBM/MFMA roofline",
            "value": a["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": a["batches"], "warmup": args.warmup,
            "ms_per_step": 1e3 * a["seconds"] / a["batches"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": "ragged24_b128", "n_layers": cfg.n_layers, "batch": cfg.batch,
                       "step": "one batch of 128: cross K/V precompute + greedy decode with forced EOS"},
            "cases": cases}))
        return
    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # one copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    res, wl = run_workload(args.workload, args.steps, args.warmup, want_roofline=True, eager=args.eager,
                           no_prefill=args.no_prefill, kv_fp8=args.kv_fp8)
    cfg = wl.cfg
    line = {
        "metric": "decoded tokens/sec at 1 MI355X (24L and 4L decoder) + % HBM/MFMA roofline",
        "value": res["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": args.workload, "kv_cache": "fp8_e4m3" if args.kv_fp8 else cfg.dtype,
                   "prompt_len": cfg.prompt_len, "max_new": cfg.max_new,
                   "enc_frames_total": int(wl.enc_lens.sum()),
                   "step": "cross K/V precompute + greedy decode of the batch",
                   "launch": "eager" if args.eager else "graph",
                   "prompt": "token by token" if args.no_prefill else "positions before the last in one pass"},
        "decode_only_tokens_per_s": res["decode_only_tokens_per_s"],
        "decode_ms_per_token_step": res["decode_ms_per_token_step"],
        "precompute_ms": res["precompute_ms"],
        "decoder_rtfx": res.get("decoder_rtfx"),
        "kernels": res.get("kernels"),
        "roofline": res.get("roofline"),
        "mfma_roofline": res.get("mfma"),
        "kernel_timing": "per kernel class: the class's launches of all layers replayed back to back between HIP events "
                         "on the decoder's stream, mid-decode state",
    }
    if not args.no_also and args.workload == "canary24_b64":
        # the 4-layer decoder at batch 256 and the large batch (1024 x 500 frames, 448 steps): their own tokens/s, the
        # attention kernels against the HBM roofline, the projection products against the MFMA roofline
        line["also"] = []
        for name, k, w in (("flash4_b256", args.steps, args.warmup), ("large24_b1024", min(args.steps, 2), min(args.warmup, 1))):
            if name == "large24_b1024" and args.no_large:
                continue
            r, _ = run_workload(name, k, w, want_roofline=True, no_prefill=args.no_prefill, kv_fp8=args.kv_fp8)
            line["also"].append({"workload": name, "value": r["tokens_per_s"], "unit": "tokens/s", "steps": k,
                                 "warmup": w, "ms_per_step": r["ms_per_step"],
                                 "decode_only_tokens_per_s": r["decode_only_tokens_per_s"],
                                 "decode_ms_per_token_step": r["decode_ms_per_token_step"],
                                 "decoder_rtfx": r.get("decoder_rtfx"), "roofline": r.get("roofline"),
                                 "attention_hbm": r.get("attention_hbm"), "mfma_projection": r.get("mfma_projection"),
                                 "mfma_roofline": r.get("mfma")})
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
