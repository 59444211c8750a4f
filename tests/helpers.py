"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI
and the oracle on the same seeded inputs and compare per-step logits."""
from __future__ import annotations

import numpy as np

from oracle import oracle as O
from paper_2307_02628_amd import skd


def run_hip(shape, w, prompts, P, N, n_min, n_max, warmup=0, mask=None, tape=None, dtype=skd.BF16,
            page_tokens=0, steps=None):
    """Prefill + teacher-forced (tape [T,B]) or free-running decode.  Returns dict like oracle.generate."""
    B = prompts.shape[0]
    steps = (N - P) if steps is None else steps
    cfg = skd.make_config(shape, B, P, N, n_min, n_max, warmup, dtype, page_tokens)
    out_logits, fed, sets = [], [], []
    with skd.Decoder(cfg, w) as dec:
        dec.prefill(prompts, mask)
        tok, lg = dec.logits_argmax()
        out_logits.append(lg)
        for k in range(steps):
            t = P + k
            sets.append(skd.skd_active_layers(t, cfg))
            if tape is None:
                fed.append(tok.copy())
                dec.decode_step(t, None)
            else:
                fed.append(np.asarray(tape[k], dtype=np.int32))
                dec.decode_step(t, fed[-1])
            tok, lg = dec.logits_argmax()
            out_logits.append(lg)
        kv = [dec.kv_len(l) for l in range(shape.L)]
        pages = dec.kv_pages()
    return {"logits": np.stack(out_logits), "fed": np.array(fed), "layers": sets, "kv_len": kv, "pages": pages}


def rel_err(got, ref):
    """max |delta logit| / (logit range), per step (axis 0)."""
    got = np.asarray(got, dtype=np.float64)
    d = np.abs(got - ref).reshape(ref.shape[0], -1).max(axis=1)
    rng = ref.reshape(ref.shape[0], -1).max(axis=1) - ref.reshape(ref.shape[0], -1).min(axis=1)
    return d / rng


def check_argmax(got_logits, ref_logits, tol, min_decided=0.5):
    """Greedy tokens must agree wherever the oracle's top-1/top-2 margin exceeds twice the logit tolerance."""
    ref = np.asarray(ref_logits)
    got = np.asarray(got_logits)
    rng = ref.max() - ref.min()
    srt = np.sort(ref, axis=-1)
    margin = srt[..., -1] - srt[..., -2]
    decided = margin > 2 * tol * rng
    assert decided.mean() >= min_decided                      # the check must not be vacuous
    np.testing.assert_array_equal(got.argmax(-1)[decided], ref.argmax(-1)[decided])


def compare(shape, w, prompts, P, N, n_min, n_max, tol, warmup=0, mask=None, dtype=skd.BF16, page_tokens=0,
            steps=None, tape=None, min_decided=0.5):
    ref = O.generate(shape, w, prompts, P, N, n_min, n_max, warmup, mask, tape=tape, steps=steps)
    got = run_hip(shape, w, prompts, P, N, n_min, n_max, warmup, mask, tape=ref["fed"], dtype=dtype,
                  page_tokens=page_tokens, steps=steps)
    assert got["layers"] == ref["layers"]                     # schedule and layer indices: exact
    assert got["kv_len"] == ref["kv_len"]                     # a layer stores exactly the columns it ran at
    err = rel_err(got["logits"], ref["logits"])
    assert err.max() <= tol, f"per-step max|dlogit|/range = {err}"
    check_argmax(got["logits"], ref["logits"], tol, min_decided)
    return got, ref, err
