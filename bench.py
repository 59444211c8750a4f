#!/usr/bin/env python3
"""Benchmark of the SkipDecode decode path on one MI355X.

One "step" = one pass of the whole hot path over one batch column:
skd_decode_step (embedding, the active layers only, KV write) followed by
skd_logits_argmax (final LayerNorm, LM head, argmax), with inputs and outputs
resident in HBM.  The default workload is the OPT-6.7B-shaped configuration
(batch 32, prompt 512, 256 decode steps, layers 32 -> 6), timed with the
SkipDecode schedule and again at full depth (n(t) = L) for the realised
speedup.  With --steps K < T the K timed steps are spread evenly over the
generation (each one timed in place during a pass over all T steps), so the
timed sample has the schedule's mean depth; both legs are repeated and the
median is reported.  The other full-size contract workloads are measured the
same way and reported under "other_workloads".  Prints ONE JSON line.
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
# the other full-size contract workloads, reported beside the default one
OTHER_WORKLOADS = ("opt1.3b_b16_p256_t256_24to12", "opt6.7b_b8_p2048_t512_32to12", "opt6.7b_b128_p64-512_t128_24to8")


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


def sample_positions(T, steps):
    """Decode steps that are timed.  All of them when steps >= T; otherwise `steps` positions spread evenly over the
    generation (the mid-points of `steps` equal strata), so that the sample's mean number of active layers and mean
    KV length are those of the whole schedule and not those of its first steps."""
    if steps >= T:
        return list(range(T))
    return [int((j + 0.5) * T / steps) for j in range(steps)]


def run_generation(skd, torch, shape, w, B, P, T, n_min, n_max, mask, steps, warmup, reps, profile, page_tokens=0,
                   warmup_layers=0, head="argmax", contiguous=False):
    """One leg (one schedule) of a workload: create a state, prefill, run the WHOLE generation once untimed (warm-up
    that also covers every launch shape), then `reps` timed repetitions.  A repetition is one more pass over the
    generation from position P in which the sampled steps (sample_positions) are each bracketed by two events on
    the library's stream: every timed step runs in its real context (cache contents, preceding step).  With
    steps >= T the whole pass sits between one pair of events instead.  `contiguous`: no untimed pass, the first
    `steps` steps are timed in one bracket after `warmup` warm-up steps (bounded dispatch count, for counter runs).
    Returns per-repetition times and the byte accounting of the timed steps."""
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

    def ev():
        return torch.cuda.Event(enable_timing=True)

    if contiguous:
        ks = list(range(min(steps, T)))
        run(0, min(warmup, T))
    else:
        ks = sample_positions(T, steps)
        run(0, T)                                   # untimed: the whole generation (>= `warmup` steps)
    dec.synchronize()
    whole = contiguous or len(ks) == T
    last = ks[-1] + 1 if contiguous else T
    rep_ms, first_ms = [], []
    for _ in range(reps):
        dec.rewind(P)
        torch.cuda.synchronize()
        if whole:
            e0, e1, f1 = ev(), ev(), ev()
            e0.record(stream)
            run(0, 1)
            f1.record(stream)
            run(1, last)
            e1.record(stream)
            torch.cuda.synchronize()
            rep_ms.append(e0.elapsed_time(e1))
            first_ms.append(e0.elapsed_time(f1))
        else:
            pairs, nxt = [], 0
            for k in sorted(set(ks) | {0}):
                run(nxt, k)
                a, b = ev(), ev()
                a.record(stream)
                run(k, k + 1)
                b.record(stream)
                pairs.append((k, a, b))
                nxt = k + 1
            run(nxt, T)
            torch.cuda.synchronize()
            t = {k: a.elapsed_time(b) for k, a, b in pairs}
            rep_ms.append(sum(t[k] for k in ks))
            first_ms.append(t[0])
    # projections of the prompt pass: 2 flops per weight and real prompt token, all L layers (attention not counted)
    prefill_flop = 2.0 * float(P * B - start.sum()) * shape.L * (4 * shape.d * shape.d + 2 * shape.d * shape.f)
    out = {"rep_ms": rep_ms, "first_step_ms": first_ms, "prefill_s": prefill_s, "ks": ks,
           "prefill_projection_pflops": prefill_flop / prefill_s / 1e15,
           "layers": [layers[k] for k in ks], "sum_len": [sum_len[k] for k in ks],
           "bytes": sum(step_bytes(shape, layers[k], sum_len[k]) for k in ks),
           "kv_pages": dec.kv_pages()}
    if profile:
        # kernel durations over the whole generation: every launch gets its own pair of events, stamped with the
        # kernel's begin and end (skd_profile_enable mode 1); then once more with event brackets around the
        # launches of each class on the stream (mode 2), which adds the cost of the two markers to every figure
        span = range(last)
        for mode, key in ((1, "profile"), (2, "profile_bracketed")):
            dec.rewind(P)
            dec.profile_enable(mode)
            run(0, last)
            prof = dec.profile_read()
            dec.profile_enable(0)
            for cls, rec in prof.items():
                if cls == "attention":
                    rec["bytes"] = sum(layers[k] * class_bytes(shape, cls, sum_len[k]) for k in span)
                elif cls == "lm_head":
                    rec["bytes"] = len(span) * class_bytes(shape, cls, 0)
                else:
                    rec["bytes"] = sum(layers[k] for k in span) * class_bytes(shape, cls, 0)
            out[key] = prof
        # step time against the number of active layers: one event pair per step of a whole pass
        dec.rewind(P)
        evs = [ev() for _ in range(last + 1)]
        evs[0].record(stream)
        for k in range(last):
            run(k, k + 1)
            evs[k + 1].record(stream)
        torch.cuda.synchronize()
        out["step_ms"] = [evs[k].elapsed_time(evs[k + 1]) for k in range(last)]
        out["step_layers"] = layers[:last]
    dec.close()
    del dec
    torch.cuda.synchronize()
    return out


def traffic_ratio(workload, kernel):
    """HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size) over algorithmic
    bytes per launch, as stored by the counter runs described in profiles/pmc_traffic_*.md.  None if that workload
    or kernel has not been measured."""
    path = os.path.join(ROOT, "profiles", "traffic_ratios.json")
    if not os.path.exists(path):
        return None
    return json.load(open(path)).get(workload, {}).get("kernels", {}).get(kernel, {}).get("ratio")


def measure_workload(skd, torch, name, w, steps, warmup, reps, profile, args):
    """Skip leg and full-depth leg of one workload; returns the figures of the bench line."""
    shape, B, P, T, n_min, n_max, ragged, *rest = WORKLOADS[name]
    wl = rest[0] if rest else 0
    steps = min(steps if steps > 0 else T, T)
    mask = S.make_ragged_mask(B, P, ragged[0], ragged[1], seed=2) if ragged else None
    skip = run_generation(skd, torch, shape, w, B, P, T, n_min, n_max, mask, steps, warmup, reps, profile,
                          args.page_tokens, wl, args.head, args.contiguous)
    full = None
    if not args.no_full_depth:
        full = run_generation(skd, torch, shape, w, B, P, T, shape.L, shape.L, mask, steps, warmup, reps, False,
                              args.page_tokens, 0, args.head, args.contiguous)
    n_timed = len(skip["ks"])
    ms = float(np.median(skip["rep_ms"]))
    tok_s = B * n_timed / (ms * 1e-3)
    gbs = skip["bytes"] / (ms * 1e-3) / 1e9
    r = np.array(skip["rep_ms"], dtype=np.float64) / n_timed
    res = {
        "value": tok_s, "unit": "tokens/s", "steps": n_timed, "ms_per_step": ms / n_timed,
        "config": {"workload": name, "batch": B, "prompt": P, "decode_steps": T,
                   "schedule": f"linear {n_max}->{n_min} of {shape.L} layers" + (f", {wl} warm-up" if wl else ""),
                   "timed_steps": ("the first %d steps" % n_timed) if args.contiguous else
                                  ("all %d steps" % T) if n_timed == T else
                                  (f"{n_timed} of {T} steps, evenly spaced (k = {', '.join(map(str, skip['ks'][:2]))}, ..., "
                                   f"{skip['ks'][-1]}), each timed inside a pass over the whole generation"),
                   "sum_n": int(sum(skip["layers"])), "mean_n": float(np.mean(skip["layers"]))},
        "hbm_gbs": gbs, "hbm_frac_of_8TBs": gbs / HBM_PEAK_GBS,
        "algorithmic_gb_per_step": skip["bytes"] / n_timed / 1e9,
        "prefill_s": skip["prefill_s"], "prefill_projection_pflops": skip["prefill_projection_pflops"],
        "kv_pages_reserved_vs_dense": list(skip["kv_pages"]),
        "ms_per_step_repeats": {"n": int(r.size), "median": float(np.median(r)), "min": float(r.min()),
                                "max": float(r.max())},
    }
    if full:
        fms = float(np.median(full["rep_ms"]))
        ftok = B * n_timed / (fms * 1e-3)
        fr = np.array(full["rep_ms"], dtype=np.float64) / n_timed
        res["full_depth"] = {"value": ftok, "unit": "tokens/s", "ms_per_step": fms / n_timed,
                             "hbm_gbs": full["bytes"] / (fms * 1e-3) / 1e9,
                             "ms_per_step_repeats": {"n": int(fr.size), "median": float(np.median(fr)),
                                                     "min": float(fr.min()), "max": float(fr.max())}}
        res["speedup_vs_full_depth"] = tok_s / ftok
        res["ideal_layer_ratio"] = shape.L * n_timed / sum(skip["layers"])
        res["ideal_byte_ratio"] = full["bytes"] / skip["bytes"]
        if n_max == shape.L and wl == 0:
            # step k = 0 runs all L layers over the same cache in both legs: the two legs on equal work
            a, b = float(np.median(skip["first_step_ms"])), float(np.median(full["first_step_ms"]))
            res["equal_depth_step_ms"] = {"skip_leg": a, "full_depth_leg": b, "ratio": b / a}
    if "step_ms" in skip:
        ns = np.array(skip["step_layers"], dtype=np.float64)
        sm = np.array(skip["step_ms"], dtype=np.float64)
        by_n = {int(n): round(float(sm[ns == n].mean()), 4) for n in sorted(set(ns.tolist()), reverse=True)}
        fit = {}
        if len(by_n) > 1:
            slope, icpt = np.polyfit(ns, sm, 1)
            resid = sm - (slope * ns + icpt)
            fit = {"ms_per_active_layer": float(slope), "ms_fixed": float(icpt),
                   "r2": float(1.0 - resid.var() / sm.var())}
        res["step_ms_by_active_layers"] = by_n
        res["step_ms_linear_fit"] = fit
    roof = None
    if "profile" in skip:
        prof = {k: v for k, v in skip["profile"].items() if v["launches"]}
        brk = skip["profile_bracketed"]
        res["kernels"] = {k: {"avg_us": 1e3 * v["ms"] / v["launches"], "launches": v["launches"],
                              "share": v["ms"] / sum(x["ms"] for x in prof.values()),
                              "gbs": (v["bytes"] / (v["ms"] * 1e-3) / 1e9) if v["bytes"] else None,
                              "avg_us_bracketed": 1e3 * brk[k]["ms"] / max(1, brk[k]["launches"])}
                          for k, v in prof.items()}
        dom = max((k for k in prof if prof[k]["bytes"]), key=lambda k: prof[k]["ms"])
        ach = prof[dom]["bytes"] / (prof[dom]["ms"] * 1e-3) / 1e9
        per_launch = prof[dom]["bytes"] / prof[dom]["launches"]
        ratio = traffic_ratio(name, dom)
        roof = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS,
                "traffic": ratio * per_launch if ratio else None,
                "traffic_source": ("HBM bytes / algorithmic bytes of this kernel on this workload as measured by "
                                   "rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (profiles/traffic_ratios.json), times "
                                   "the algorithmic bytes per launch of this run") if ratio else None,
                "bytes_per_launch": per_launch,
                "avg_launch_us": 1e3 * prof[dom]["ms"] / prof[dom]["launches"],
                "launches": prof[dom]["launches"],
                "duration": "begin/end time stamps of every launch of this kernel over all decode steps of the "
                            "workload (HIP events attached to the launch), skip schedule",
                "frac_with_event_brackets": brk[dom]["bytes"] / (brk[dom]["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
    res["roofline"] = roof
    return res


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
    ap.add_argument("--steps", type=int, default=0,
                    help="decode steps to time (default: the workload's T); fewer than T = that many steps spread "
                         "evenly over the generation")
    ap.add_argument("--warmup", type=int, default=8,
                    help="untimed warm-up steps (the untimed pass over the whole generation always covers them)")
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed region (the line reports the median)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="only the named workload (default: the other contract workloads are measured as well)")
    ap.add_argument("--no-table2-presets", action="store_true",
                    help="skip the paper's Table 2 presets (default: measured at the contract batch and lengths)")
    ap.add_argument("--contiguous", action="store_true",
                    help="time the FIRST --steps steps in one bracket, with no pass over the whole generation "
                         "(bounded number of launches: for hardware-counter runs)")
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
    weights = {}

    def weights_of(sh):
        if sh not in weights:
            weights.clear()              # one model's weights resident at a time
            torch.cuda.empty_cache()
            weights[sh] = device_weights(sh, 0)
        return weights[sh]

    # The other contract workloads (same measurement, fewer repetitions), and Table 2's eight presets (warm-up layer,
    # min and max layer per target speed-up) at the batch and lengths of the contract workload with the same model
    # shape, whose full-depth leg is theirs as well (same shapes, n = L everywhere).  One model's weights are resident
    # at a time: everything of the default workload's shape first.
    others, presets = {}, {}
    want_others = not args.no_other_workloads and args.workload == DEFAULT_WORKLOAD
    want_presets = want_others and not args.no_table2_presets and not args.no_full_depth

    class _SkipLegOnly:
        pass
    pa = _SkipLegOnly()
    pa.__dict__.update(vars(args))
    pa.no_full_depth = True

    def other(name):
        o = measure_workload(skd, torch, name, weights_of(WORKLOADS[name][0]), args.steps, args.warmup,
                             max(3, args.reps // 2 + 1), not args.no_profile, args)
        keep = ("value", "unit", "steps", "ms_per_step", "hbm_gbs", "hbm_frac_of_8TBs", "algorithmic_gb_per_step",
                "prefill_s", "prefill_projection_pflops", "speedup_vs_full_depth", "ideal_layer_ratio", "ideal_byte_ratio",
                "ms_per_step_repeats", "equal_depth_step_ms")
        others[name] = {k: o[k] for k in keep if k in o}
        others[name]["config"] = o["config"]
        if "full_depth" in o:
            others[name]["full_depth"] = {k: o["full_depth"][k] for k in ("value", "ms_per_step")}
        if o.get("roofline"):
            others[name]["roofline"] = {k: o["roofline"][k] for k in ("kernel", "achieved", "frac", "traffic",
                                                                      "bytes_per_launch", "avg_launch_us")}
        if "kernels" in o:
            others[name]["kernels_gbs"] = {k: (round(v["gbs"], 1) if v["gbs"] else None)
                                           for k, v in o["kernels"].items()}
            others[name]["kernels_avg_us"] = {k: round(v["avg_us"], 2) for k, v in o["kernels"].items()}

    def preset(name, full_depth_tok_s):
        sh, _B, _P, _T, lo, hi, _r, wl_ = WORKLOADS[name]
        o = measure_workload(skd, torch, name, weights_of(sh), args.steps, args.warmup, 3, False, pa)
        presets[name] = {"target_speedup": int(name.rsplit("-", 1)[1][0]), "warmup_min_max_layers": [wl_, lo, hi],
                         "value": o["value"], "unit": "tokens/s", "ms_per_step": o["ms_per_step"],
                         "hbm_frac_of_8TBs": o["hbm_frac_of_8TBs"], "mean_n": o["config"]["mean_n"],
                         "speedup_vs_full_depth": o["value"] / full_depth_tok_s,
                         "ideal_layer_ratio": sh.L / o["config"]["mean_n"]}

    # Order: the small model first, on a fresh device (measured: its step is 3 % slower when its buffers are carved
    # out of what the 13 GB states of the large model left behind), then everything of the 6.7B shape.
    if want_others:
        for name in OTHER_WORKLOADS:
            if WORKLOADS[name][0] != shape:
                other(name)
        base13 = others.get("opt1.3b_b16_p256_t256_24to12", {}).get("full_depth", {}).get("value")
        if want_presets and base13:
            for name in sorted(n for n in WORKLOADS if n.startswith("opt1.3b_b16_p256_t256_table2-")):
                preset(name, base13)
    m = measure_workload(skd, torch, args.workload, weights_of(shape), args.steps, args.warmup, args.reps,
                         not args.no_profile, args)
    res = {
        "metric": "generated tokens/sec at OPT-6.7B shape, B=32, skip vs full depth; HBM GB/s",
        "value": m.pop("value"), "unit": m.pop("unit"), "n_gpus": 1, "steps": m.pop("steps"), "warmup": args.warmup,
        "ms_per_step": m.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "head": args.head,
        "config": m.pop("config"), "device_copy_read_plus_write_gbs": copy_gbs,
    }
    res.update(m)
    if want_others:
        for name in OTHER_WORKLOADS:
            if WORKLOADS[name][0] == shape:
                other(name)
        if want_presets and "full_depth" in res:
            for name in sorted(n for n in WORKLOADS if n.startswith("opt6.7b_b32_p512_t256_table2-")):
                preset(name, res["full_depth"]["value"])
    weights.clear()
    torch.cuda.empty_cache()
    if others:
        res["other_workloads"] = others
    if presets:
        res["table2_presets"] = presets
    res["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(shape, B, P, T, n_min, n_max)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
