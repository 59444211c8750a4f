#!/usr/bin/env python3
"""Benchmark of the SkipDecode decode path on one MI355X.

One "step" = one pass of the whole hot path over one batch column:
skd_decode_step (embedding, the active layers only, KV write) followed by
skd_logits_argmax (final LayerNorm, LM head, argmax), with inputs and outputs
resident in HBM.  The default workload is the OPT-6.7B-shaped configuration
(batch 32, prompt 512, 256 decode steps, layers 32 -> 6), timed with the
SkipDecode schedule and again at full depth (n(t) = L) for the realised
speedup.  Prints ONE JSON line.
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

import synth_inputs as S  # noqa: E402

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published

# Table 2 of the paper: (warm-up layers, min layer, max layer) per target speed-up
TABLE2 = {"opt6.7b": {2: (1, 11, 22), 3: (1, 8, 14), 4: (1, 6, 10), 5: (1, 5, 8)},
          "opt1.3b": {2: (1, 8, 16), 3: (1, 6, 10), 4: (1, 5, 7), 5: (1, 4, 6)}}

WORKLOADS = {
    # name: (shape, B, P, T, n_min, n_max, ragged prompt lengths or None[, warm-up layers])
    "opt1.3b_b16_p256_t256_24to12": (S.OPT_1_3B, 16, 256, 256, 12, 24, None),
    "opt6.7b_b32_p512_t256_32to6": (S.OPT_6_7B, 32, 512, 256, 6, 32, None),
    "opt6.7b_b8_p2048_t512_32to12": (S.OPT_6_7B, 8, 2048, 512, 12, 32, None),
    "opt6.7b_b128_p64-512_t128_24to8": (S.OPT_6_7B, 128, 512, 128, 8, 24, (64, 512)),
    "tiny_b2_p16_t16_4to2": (S.TINY, 2, 16, 16, 2, 4, None),
    # two layers of the 6.7B shape with the primary workload's batch and lengths: same per-launch kernel shapes,
    # short enough for counter collection
    "opt6.7b-2layers_b32_p512_t256_2to1": (S.ModelShape(2, 4096, 32, 16384, 50272, 3072), 32, 512, 256, 1, 2, None),
    "opt6.7b-2layers_b128_p64-512_t128_2to1": (S.ModelShape(2, 4096, 32, 16384, 50272, 3072), 128, 512, 128, 1, 2,
                                                (64, 512)),
}
for _x, (_w, _lo, _hi) in TABLE2["opt6.7b"].items():   # the paper's presets at the primary workload's batch and lengths
    WORKLOADS[f"opt6.7b_b32_p512_t256_table2-{_x}x"] = (S.OPT_6_7B, 32, 512, 256, _lo, _hi, None, _w)
for _x, (_w, _lo, _hi) in TABLE2["opt1.3b"].items():
    WORKLOADS[f"opt1.3b_b16_p256_t256_table2-{_x}x"] = (S.OPT_1_3B, 16, 256, 256, _lo, _hi, None, _w)
DEFAULT_WORKLOAD = "opt6.7b_b32_p512_t256_32to6"


def device_weights(shape, seed=0):
    """Random-init bf16 weights N(0, 0.02) generated directly in HBM (LayerNorm gains around 1)."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)

    def rnd(*sz, mean=0.0):
        return (torch.randn(*sz, generator=g, device="cuda", dtype=torch.float32) * 0.02 + mean).to(torch.bfloat16)

    w = {"tok_emb": rnd(shape.V, shape.d), "pos_emb": rnd(shape.max_pos, shape.d),
         "lnf_g": rnd(shape.d, mean=1.0), "lnf_b": rnd(shape.d)}
    shapes = S.layer_tensor_shapes(shape)
    for name, sz in shapes.items():
        mean = 1.0 if name in ("ln1_g", "ln2_g") else 0.0
        w[name] = [rnd(*sz, mean=mean) for _ in range(shape.L)]
    return w


def step_bytes(shape, n_layers, sum_len):
    """Algorithmic HBM bytes of one decode step: weights of the active layers, the valid KV entries they read,
    and the LM head (bf16 = 2 bytes; vectors counted in fp32 as stored)."""
    d, f, V = shape.d, shape.f, shape.V
    per_layer_w = 2 * (3 * d * d + d * d + 2 * d * f) + 4 * (3 * d + d + f + d + 4 * d)
    per_layer_kv = 2 * 2 * d * sum_len
    return n_layers * (per_layer_w + per_layer_kv) + 2 * V * d


def class_bytes(shape, cls, sum_len):
    d, f, V = shape.d, shape.f, shape.V
    return {"gemm_qkv": 2 * 3 * d * d, "gemm_out": 2 * d * d, "gemm_ffn1": 2 * d * f, "gemm_ffn2": 2 * d * f,
            "lm_head": 2 * V * d, "attention": 2 * 2 * d * sum_len}.get(cls, 0)


def run_generation(skd, torch, shape, w, B, P, T, n_min, n_max, mask, steps, warmup, profile, page_tokens=0,
                   warmup_layers=0, head="argmax"):
    """Create a state, prefill, warm up, rewind, time `steps` decode steps.  Returns timing dict."""
    N = P + T
    stream = torch.cuda.Stream()
    cfg = skd.make_config(shape, B, P, N, n_min, n_max, warmup_layers, dtype=skd.BF16, io_on_device=1,
                          page_tokens=page_tokens)
    g = torch.Generator(device="cpu")
    g.manual_seed(1)
    prompts = torch.randint(0, shape.V, (P, B), generator=g, dtype=torch.int32).cuda()      # [P][B]
    tape = torch.randint(0, shape.V, (T, B), generator=g, dtype=torch.int32).cuda()         # teacher-forced inputs
    toks = torch.zeros(B, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    dec = skd.Decoder(cfg, w, location=skd.DEVICE, elem=skd.W_BF16, stream=stream.cuda_stream)
    t0 = time.time()
    dec.prefill(prompts, mask)
    dec.synchronize()
    prefill_s = time.time() - t0
    layers = [len(skd.skd_active_layers(P + k, cfg)) for k in range(T)]
    start = np.zeros(B, dtype=np.int64) if mask is None else (mask == 0).sum(axis=1)
    sum_len = [int((P + k + 1) * B - start.sum()) for k in range(T)]

    uni = torch.rand((T, B), generator=g, dtype=torch.float32).clamp_(0.0, 0.999999).cuda()

    def run(k0, k1):
        for k in range(k0, k1):
            dec.decode_step(P + k, tape[k])
            if head == "sample":
                dec.logits_sample_device(uni[k], 0.3, 0.7, toks, None)
            else:
                dec.logits_argmax_device(toks, None)

    run(0, min(warmup, T))
    dec.synchronize()
    dec.rewind(P)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record(stream)
    run(0, steps)
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1)
    out = {"ms": ms, "prefill_s": prefill_s, "layers": layers[:steps], "sum_len": sum_len[:steps],
           "bytes": sum(step_bytes(shape, layers[k], sum_len[k]) for k in range(steps)),
           "kv_pages": dec.kv_pages()}
    if profile:
        # the same timed region four more times (the line's `value` stays the first, contract-defined one)
        reps = [ms]
        for _ in range(4):
            dec.rewind(P)
            torch.cuda.synchronize()
            ev0.record(stream)
            run(0, steps)
            ev1.record(stream)
            torch.cuda.synchronize()
            reps.append(ev0.elapsed_time(ev1))
        out["repeat_ms"] = reps
        dec.rewind(P)
        dec.profile_enable(True)
        run(0, steps)
        prof = dec.profile_read()
        dec.profile_enable(False)
        for cls, rec in prof.items():
            if cls == "attention":
                rec["bytes"] = sum(layers[k] * class_bytes(shape, cls, sum_len[k]) for k in range(steps))
            elif cls == "lm_head":
                rec["bytes"] = steps * class_bytes(shape, cls, 0)
            else:
                rec["bytes"] = sum(layers[:steps]) * class_bytes(shape, cls, 0)
        out["profile"] = prof
        # step time against the number of active layers: one event pair per step
        dec.rewind(P)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        evs[0].record(stream)
        for k in range(steps):
            run(k, k + 1)
            evs[k + 1].record(stream)
        torch.cuda.synchronize()
        out["step_ms"] = [evs[k].elapsed_time(evs[k + 1]) for k in range(steps)]
    dec.close()
    del dec
    torch.cuda.synchronize()
    return out


def cpu_baseline(shape, B, P, T, n_min, n_max):
    """Time the fp32 build of the oracle on a bounded sample of the same workload: three complete decode steps
    (all B rows, the true layer sets, KV caches of the true lengths filled with synthetic values, final LayerNorm +
    LM head + argmax) at the quarter points of the generation."""
    from oracle import oracle as O
    N = P + T
    ks = sorted({max(0, T // 4), T // 2, min(T - 1, (3 * T) // 4)})
    distinct = 2                                   # layer weight sets alternated over the stack (values do not matter)
    w = S.make_weights(shape, seed=0, layers=distinct)
    wl = {key: ([val[l % distinct] for l in range(shape.L)] if isinstance(val, list) else val) for key, val in w.items()}
    g = np.random.Generator(np.random.Philox(key=[11, 1]))
    kv_full = g.standard_normal(size=(B, P + ks[-1], shape.d), dtype=np.float32) * np.float32(0.5)
    tok = S.make_token_tape(B, 1, shape.V, seed=3)[0]
    total, parts = 0.0, []
    for k in ks:
        t = P + k
        layers = O.active_layers(t, P, N, n_min, n_max, 0, shape.L, "f32")
        dec = O.Decoder(shape, wl, B, N, "f32")
        kv = np.ascontiguousarray(kv_full[:, :t])
        for l in layers:
            dec.kv_load(l, kv, kv)
        dec.seek(t)
        t0 = time.time()
        dec.column(t, tok, layers, want_logits=True)
        sec = time.time() - t0
        dec.close()
        total += sec
        parts.append(f"k={k} (position {t}, {len(layers)} layers) {sec:.2f} s")
    return {"value": B * len(ks) / total, "unit": "tokens/s", "cores": O.threads("f32"), "kind": "oracle",
            "sample": f"{len(ks)} full decode steps of the workload (all {B} rows, true layer sets, synthetic KV of the "
                      f"true lengths, LM head + argmax), fp32 oracle build: " + "; ".join(parts)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (default: the workload's T)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--no-full-depth", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--page-tokens", type=int, default=0, help="KV page size in tokens (0 = library default)")
    ap.add_argument("--head", choices=["argmax", "sample"], default="argmax",
                    help="token head after the LM head: greedy argmax (contract) or temperature 0.3 / top-p 0.7 sampling")
    ap.add_argument("--calib-copy", action="store_true",
                    help="first run a plain 1 GiB device copy 4 times (reference kernel of known traffic for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2307_02628_amd import _build, skd
    if not os.path.exists(skd.LIB_PATH):
        _build.build(force=True)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # context for the roofline fractions: what a plain library copy reaches on this machine (bytes read + written)
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dst.copy_(src)
    e0.record()
    for _ in range(4):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 4 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()

    shape, B, P, T, n_min, n_max, ragged, *rest = WORKLOADS[args.workload]
    wl = rest[0] if rest else 0
    steps = args.steps if args.steps > 0 else T
    steps = min(steps, T)
    mask = None
    if ragged:
        mask = S.make_ragged_mask(B, P, ragged[0], ragged[1], seed=2)
    w = device_weights(shape, 0)
    skip = run_generation(skd, torch, shape, w, B, P, T, n_min, n_max, mask, steps, args.warmup, not args.no_profile, args.page_tokens, wl, args.head)
    full = None
    if not args.no_full_depth:
        full = run_generation(skd, torch, shape, w, B, P, T, shape.L, shape.L, mask, steps, args.warmup, False, args.page_tokens)
    del w
    torch.cuda.empty_cache()

    tok_s = B * steps / (skip["ms"] * 1e-3)
    gbs = skip["bytes"] / (skip["ms"] * 1e-3) / 1e9
    res = {
        "metric": "generated tokens/sec at OPT-6.7B shape, B=32, skip vs full depth; HBM GB/s",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": skip["ms"] / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "head": args.head,
        "config": {"workload": args.workload, "batch": B, "prompt": P, "decode_steps": T,
                   "schedule": f"linear {n_max}->{n_min} of {shape.L} layers" + (f", {wl} warm-up" if wl else ""),
                   "sum_n": int(sum(skip["layers"]))},
        "hbm_gbs": gbs, "hbm_frac_of_8TBs": gbs / HBM_PEAK_GBS, "device_copy_read_plus_write_gbs": copy_gbs,
        "algorithmic_gb_per_step": skip["bytes"] / steps / 1e9,
        "prefill_s": skip["prefill_s"],
        "kv_pages_reserved_vs_dense": list(skip["kv_pages"]),
    }
    if full:
        ftok = B * steps / (full["ms"] * 1e-3)
        res["full_depth"] = {"value": ftok, "unit": "tokens/s", "ms_per_step": full["ms"] / steps,
                             "hbm_gbs": full["bytes"] / (full["ms"] * 1e-3) / 1e9}
        res["speedup_vs_full_depth"] = tok_s / ftok
        res["ideal_layer_ratio"] = shape.L * steps / sum(skip["layers"])
        res["ideal_byte_ratio"] = full["bytes"] / skip["bytes"]
    if "repeat_ms" in skip:
        r = np.array(skip["repeat_ms"], dtype=np.float64) / steps
        res["ms_per_step_repeats"] = {"n": int(r.size), "median": float(np.median(r)), "min": float(r.min()),
                                      "max": float(r.max())}
    if "step_ms" in skip:
        ns = np.array(skip["layers"], dtype=np.float64)
        ms = np.array(skip["step_ms"], dtype=np.float64)
        by_n = {int(n): round(float(ms[ns == n].mean()), 4) for n in sorted(set(ns.tolist()), reverse=True)}
        fit = {}
        if len(by_n) > 1:
            slope, icpt = np.polyfit(ns, ms, 1)
            resid = ms - (slope * ns + icpt)
            fit = {"ms_per_active_layer": float(slope), "ms_fixed": float(icpt),
                   "r2": float(1.0 - resid.var() / ms.var())}
        res["step_ms_by_active_layers"] = by_n
        res["step_ms_linear_fit"] = fit
    roof = None
    if "profile" in skip:
        prof = {k: v for k, v in skip["profile"].items() if v["launches"]}
        res["kernels"] = {k: {"avg_us": 1e3 * v["ms"] / v["launches"], "launches": v["launches"],
                              "share": v["ms"] / sum(x["ms"] for x in prof.values()),
                              "gbs": (v["bytes"] / (v["ms"] * 1e-3) / 1e9) if v["bytes"] else None}
                          for k, v in prof.items()}
        dom = max((k for k in prof if prof[k]["bytes"]), key=lambda k: prof[k]["ms"])
        ach = prof[dom]["bytes"] / (prof[dom]["ms"] * 1e-3) / 1e9
        # HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE: the ratio to the algorithmic bytes was
        # measured per kernel on a 2-layer slice with the same launch shapes (profiles/pmc_traffic_*.md)
        traffic = None
        tfile = os.path.join(ROOT, "profiles", "traffic_ratios_opt6.7b_b32.json")
        if os.path.exists(tfile) and shape.d == 4096 and B == 32:
            ratio = json.load(open(tfile))["kernels"].get(dom, {}).get("ratio")
            if ratio:
                traffic = ratio * prof[dom]["bytes"] / prof[dom]["launches"]
        roof = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
                "bytes_per_launch": prof[dom]["bytes"] / prof[dom]["launches"],
                "avg_launch_us": 1e3 * prof[dom]["ms"] / prof[dom]["launches"]}
    res["roofline"] = roof
    res["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(shape, B, P, T, n_min, n_max)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
