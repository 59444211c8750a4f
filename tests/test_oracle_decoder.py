"""Pins for the oracle's decoder (cached column-wise form and brute-force form).

Independent reference: `torch_prefix_decoder` below assembles the decoder from
PyTorch CPU library routines in float64 (layer_norm, linear, softmax, matmul)
over whole sequences with a causal mask -- the textbook pre-LayerNorm decoder.
It shares no code with the oracle.  Skipping enters it only through the fact
the paper derives in Section 2.2: with monotonically decreasing exits, the
columns at which a layer runs are a prefix of the sequence, so "layer l" is an
ordinary causal transformer block applied to that prefix.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as S
from oracle import oracle as O

SMALL = S.ModelShape(L=4, d=32, H=4, f=64, V=50, max_pos=32)


def torch_prefix_decoder(shape, w, tokens, prefix_len, mask=None):
    """tokens [B,C]; prefix_len[l] = number of leading columns layer l processes.
    Returns logits [B,C,V] (float64) of every column."""
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    tok = torch.from_numpy(np.asarray(tokens, dtype=np.int64))
    B, C = tok.shape
    real = torch.ones(B, C, dtype=torch.bool) if mask is None else torch.from_numpy(np.asarray(mask) != 0)
    pos = torch.cumsum(real.long(), dim=1) - real.long()          # real tokens before each column
    h = t64(w["tok_emb"])[tok] + t64(w["pos_emb"])[pos]
    for l in range(shape.L):
        c = int(prefix_len[l])
        if c == 0:
            continue
        x = h[:, :c]
        a = F.layer_norm(x, (shape.d,), t64(w["ln1_g"][l]), t64(w["ln1_b"][l]), eps=1e-5)
        qkv = F.linear(a, t64(w["wqkv"][l]), t64(w["bqkv"][l]))
        q, k, v = qkv.split(shape.d, dim=-1)
        sp = lambda z: z.reshape(B, c, shape.H, shape.dh).transpose(1, 2)       # [B,H,c,dh]
        s = torch.matmul(sp(q), sp(k).transpose(-1, -2)) / (shape.dh ** 0.5)
        allow = torch.tril(torch.ones(c, c, dtype=torch.bool))[None, None] & real[:, None, None, :c]
        s = s.masked_fill(~allow, float("-inf"))
        p = torch.softmax(s, dim=-1)
        p = torch.nan_to_num(p, nan=0.0)                          # rows with no allowed key (pads)
        o = torch.matmul(p, sp(v)).transpose(1, 2).reshape(B, c, shape.d)
        x = x + F.linear(o, t64(w["wo"][l]), t64(w["bo"][l]))
        m = F.layer_norm(x, (shape.d,), t64(w["ln2_g"][l]), t64(w["ln2_b"][l]), eps=1e-5)
        x = x + F.linear(F.relu(F.linear(m, t64(w["w1"][l]), t64(w["b1"][l]))), t64(w["w2"][l]), t64(w["b2"][l]))
        h = torch.cat([x, h[:, c:]], dim=1)
    y = F.layer_norm(h, (shape.d,), t64(w["lnf_g"]), t64(w["lnf_b"]), eps=1e-5)
    head = w.get("lm_head")
    return F.linear(y, t64(w["tok_emb"] if head is None else head)).numpy()


def layer_sets(shape, P, N, n_min, n_max, warmup=0):
    return [O.active_layers(i, P, N, n_min, n_max, warmup, shape.L) for i in range(N)]


def prefix_lengths(shape, sets):
    on = np.zeros((len(sets), shape.L), dtype=bool)
    for i, A in enumerate(sets):
        on[i, A] = True
    pl = on.sum(axis=0)
    for l in range(shape.L):                                       # must really be prefixes
        assert on[:pl[l], l].all() and not on[pl[l]:, l].any()
    return pl


def run_cached(shape, w, tokens, sets, mask=None, real="f64"):
    """Feed the token matrix column by column; returns logits [B,C,V]."""
    B, C = tokens.shape
    dec = O.Decoder(shape, w, B, C, real)
    out = []
    for i in range(C):
        rt = None if mask is None else mask[:, i]
        lg, _ = dec.column(i, tokens[:, i], sets[i], rt)
        out.append(lg)
    kv = [dec.kv_len(l) for l in range(shape.L)]
    dec.close()
    return np.stack(out, axis=1), kv


def test_full_depth_equals_textbook_decoder():
    # Section 3.1: besides the skipping policy nothing in the transformer
    # changes, so n(i) = L everywhere must be ordinary decoding.
    w = S.make_weights(SMALL, seed=3)
    tok = S.make_prompts(3, 12, SMALL.V, seed=4)
    ref = torch_prefix_decoder(SMALL, w, tok, [12] * SMALL.L)
    got, kv = run_cached(SMALL, w, tok, [list(range(SMALL.L))] * 12)
    assert kv == [12] * SMALL.L
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_tiny_contract_config_full_depth():
    w = S.make_weights(S.TINY, seed=0)
    tok = S.make_prompts(2, 10, S.TINY.V, seed=1)
    ref = torch_prefix_decoder(S.TINY, w, tok, [10] * S.TINY.L)
    got, _ = run_cached(S.TINY, w, tok, [list(range(S.TINY.L))] * 10)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11)


@pytest.mark.parametrize("n_min,n_max,warmup,P,N", [
    (2, 4, 0, 5, 12),      # config-1 style 4 -> 2
    (1, 4, 0, 3, 12),      # down to a single layer
    (1, 3, 0, 4, 7),       # n_max < L and drops of more than one layer per step
    (2, 3, 1, 4, 12),      # one warm-up layer + top window
    (2, 2, 2, 2, 6),       # warm-up uses the whole budget
])
def test_skip_equals_prefix_form_and_bruteforce(n_min, n_max, warmup, P, N):
    w = S.make_weights(SMALL, seed=5)
    tok = S.make_prompts(2, N, SMALL.V, seed=6)
    sets = layer_sets(SMALL, P, N, n_min, n_max, warmup)
    pl = prefix_lengths(SMALL, sets)
    ref = torch_prefix_decoder(SMALL, w, tok, pl)
    got, kv = run_cached(SMALL, w, tok, sets)
    # cache lengths: a layer holds exactly the columns at which it ran
    assert kv == [int(x) for x in pl]
    assert sum(kv) == sum(len(A) for A in sets)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    # brute force without any cache, layer-major loop order
    on = np.zeros((N, SMALL.L), dtype=np.uint8)
    for i, A in enumerate(sets):
        on[i, A] = 1
    for C in (1, P, P + 1, N - 1, N):
        bf = O.recompute(SMALL, w, tok[:, :C], on[:C])
        np.testing.assert_allclose(bf, got[:, C - 1], rtol=0, atol=1e-12)


def test_left_padding_matches_unpadded_row():
    # A row of true length p inside a left-padded batch must decode exactly
    # like the same row alone and unpadded (schedule depends on the step
    # index and T only).
    w = S.make_weights(SMALL, seed=8)
    P, T = 8, 6
    N = P + T
    mask = S.make_ragged_mask(3, P, 2, 8, seed=9)
    mask[0, :] = 1                                                 # one full row
    tok = S.make_prompts(3, N, SMALL.V, seed=10)
    sets = layer_sets(SMALL, P, N, 2, 4)
    full_mask = np.concatenate([mask, np.ones((3, T), np.uint8)], axis=1)
    got, _ = run_cached(SMALL, w, tok, sets, full_mask)
    ref = torch_prefix_decoder(SMALL, w, tok, prefix_lengths(SMALL, sets), full_mask)
    real = full_mask.astype(bool)
    np.testing.assert_allclose(got[real], ref[real], rtol=0, atol=1e-12)
    for b in range(3):
        p = int(mask[b].sum())
        alone = tok[b:b + 1, P - p:]
        sets_b = layer_sets(SMALL, p, p + T, 2, 4)
        got_b, _ = run_cached(SMALL, w, alone, sets_b)
        np.testing.assert_allclose(got_b[0], got[b, P - p:], rtol=0, atol=1e-12)
        bf = O.recompute(SMALL, w, tok[b:b + 1], np.array([[l in A for l in range(SMALL.L)] for A in sets]),
                         full_mask[b:b + 1])
        np.testing.assert_allclose(bf[0], got[b, -1], rtol=0, atol=1e-12)


def test_batch_invariance():
    # Section 2.1: one exit point per column for all rows; rows do not interact.
    w = S.make_weights(SMALL, seed=11)
    tok = S.make_prompts(3, 10, SMALL.V, seed=12)
    sets = layer_sets(SMALL, 4, 10, 1, 4)
    got, _ = run_cached(SMALL, w, tok, sets)
    for b in range(3):
        one, _ = run_cached(SMALL, w, tok[b:b + 1], sets)
        np.testing.assert_array_equal(one[0], got[b])


def test_skipped_layers_are_dead_and_top_layers_matter():
    # Section 2.4: the budget goes to the top layers.  After the prompt, with
    # n_max = 2 of L = 4, layers 0 and 1 never run again: overwriting their
    # weights with garbage once the prompt is done cannot change any decode
    # logit, while touching a top layer does.
    P, N = 4, 10
    w = S.make_weights(SMALL, seed=13)
    tok = S.make_prompts(2, N, SMALL.V, seed=14)
    sets = layer_sets(SMALL, P, N, 1, 2)
    assert all(min(A) >= 2 for A in sets[P:])
    base, _ = run_cached(SMALL, w, tok, sets)

    def decode_after_damage(names, layers, value):
        w2 = {k: ([x.copy() for x in v] if isinstance(v, list) else v.copy()) for k, v in w.items()}
        dec = O.Decoder(SMALL, w2, 2, N)
        for i in range(P):
            dec.column(i, tok[:, i], sets[i], want_logits=False)
        for name in names:                      # the decoder reads these very arrays
            for l in layers:
                w2[name][l][...] = value
        out = [dec.column(i, tok[:, i], sets[i])[0] for i in range(P, N)]
        dec.close()
        return np.stack(out, axis=1)

    every = ("wqkv", "wo", "w1", "w2", "bqkv", "bo", "b1", "b2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")
    np.testing.assert_array_equal(decode_after_damage(every, (0, 1), 7.5), base[:, P:])
    assert np.abs(decode_after_damage(("w2",), (3,), 0.01) - base[:, P:]).max() > 1e-3
    assert np.abs(decode_after_damage(("bqkv",), (2,), 0.3) - base[:, P:]).max() > 1e-3


def test_non_monotone_layer_sets_are_refused():
    w = S.make_weights(SMALL, seed=15)
    tok = S.make_prompts(1, 4, SMALL.V, seed=16)
    dec = O.Decoder(SMALL, w, 1, 4)
    dec.column(0, tok[:, 0], [0, 1, 2, 3])
    dec.column(1, tok[:, 1], [2, 3])
    rc, _, _ = dec.column_rc(2, tok[:, 2], [1, 2, 3])              # layer 1 lacks column 1
    assert rc == O.ERR_ORDER
    rc, _, _ = dec.column_rc(2, tok[:, 2], [3, 2])                 # not ascending
    assert rc == O.ERR_SCHEDULE
    rc, _, _ = dec.column_rc(3, tok[:, 3], [3])                    # columns must come in order
    assert rc == O.ERR_ORDER
    dec.close()
    on = np.array([[1, 1, 1, 1], [0, 0, 1, 1], [0, 1, 1, 1], [0, 0, 0, 1]], np.uint8)
    rc, _ = O.recompute_rc(SMALL, w, tok, on)
    assert rc == O.ERR_SCHEDULE


def test_generate_contract_config_1():
    # Tiny contract configuration: L=4, batch 2, prompt 16, 16 decode steps, 4 -> 2.
    w = S.make_weights(S.TINY, seed=0)
    pr = S.make_prompts(2, 16, S.TINY.V, seed=1)
    r = O.generate(S.TINY, w, pr, 16, 32, 2, 4)
    assert [len(A) for A in r["layers"]] == [4] * 5 + [3] * 8 + [2] * 3
    assert sum(len(A) for A in r["layers"]) == 50
    assert r["kv_len"] == [16 + 5, 16 + 13, 32, 32]
    assert sum(r["kv_len"]) == 16 * 4 + 50                         # P*L + sum n : no entry is ever recomputed
    # greedy free-running: the token fed at step k is the argmax of step k-1's logits
    for k in range(16):
        np.testing.assert_array_equal(r["fed"][k], r["logits"][k].argmax(axis=1))
    # the same tokens, teacher-forced, reproduce the same logits; and the
    # fp32 build of the oracle stays close to the fp64 one
    r2 = O.generate(S.TINY, w, pr, 16, 32, 2, 4, tape=r["fed"])
    np.testing.assert_array_equal(r2["logits"], r["logits"])
    r3 = O.generate(S.TINY, w, pr, 16, 32, 2, 4, tape=r["fed"], real="f32")
    rng = r["logits"].max() - r["logits"].min()
    assert np.abs(r3["logits"] - r["logits"]).max() / rng < 1e-5


def test_ops_against_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 48))
    g, b = rng.standard_normal(48).astype(np.float32), rng.standard_normal(48).astype(np.float32)
    ref = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g).double(), torch.from_numpy(b).double(), 1e-5)
    np.testing.assert_allclose(O.op_layernorm(x, g, b), ref.numpy(), atol=1e-12)
    W = rng.standard_normal((7, 48)).astype(np.float32)
    bias = rng.standard_normal(7).astype(np.float32)
    np.testing.assert_allclose(O.op_linear(W, bias, x), x @ W.astype(np.float64).T + bias, atol=1e-12)
    H, dh, ln = 3, 16, 9
    q, K, V = rng.standard_normal(48), rng.standard_normal((ln, 48)), rng.standard_normal((ln, 48))
    valid = np.array([0, 1, 1, 0, 1, 1, 1, 1, 1], np.uint8)
    out = O.op_attention(q, K, V, H, valid)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        s = (K[:, sl] @ q[sl]) / np.sqrt(dh)
        s[valid == 0] = -np.inf
        p = torch.softmax(torch.from_numpy(s), 0).numpy()
        np.testing.assert_allclose(out[sl], p @ V[:, sl], atol=1e-12)


def test_sampling_head_pins():
    # Section 3.2 generation setting (temperature, top-p): hand-computed cases, limits and the library softmax.
    lg = np.log(np.array([0.5, 0.3, 0.2]))
    # nucleus for top_p 0.7 is {0, 1} (0.5 alone is short of 0.7); running sums 0.5, 0.8 over a mass of 0.8
    assert O.op_sample(lg, 1.0, 0.7, 0.50)[0] == 0          # 0.5 * 0.8 = 0.40 < 0.5
    assert O.op_sample(lg, 1.0, 0.7, 0.63)[0] == 1          # 0.504 > 0.5
    assert O.op_sample(lg, 1.0, 0.7, 0.999)[0] == 1         # token 2 is outside the nucleus
    assert O.op_sample(lg, 1.0, 0.5, 0.999)[0] == 0         # 0.5 reaches top_p = 0.5 on its own
    assert O.op_sample(lg, 1.0, 1.0, 0.999)[0] == 2         # everything is in
    assert O.op_sample(lg, 0.01, 1.0, 0.999)[0] == 0        # temperature -> 0 is the argmax
    # ties with the last admitted value are admitted too: [0.4, 0.3, 0.3], top_p 0.6 -> all three
    tie = np.log(np.array([0.4, 0.3, 0.3]))
    assert O.op_sample(tie, 1.0, 0.6, 0.95)[0] == 2
    # top_p = 1: plain inverse-CDF sampling of softmax(z / T), against the library softmax
    rng = np.random.default_rng(3)
    z = rng.standard_normal(500) * 2
    for T in (0.3, 1.0, 1.7):
        p = torch.softmax(torch.from_numpy(z / T), 0).numpy()
        cdf = np.cumsum(p)
        for u in rng.random(50):
            tok, _, m = O.op_sample(z, T, 1.0, float(u))
            if m > 1e-9:
                assert tok == int(np.searchsorted(cdf, u, side="right"))
    # with top_p < 1 the sample always lies in the smallest top set reaching top_p, and its frequency follows the
    # renormalised probabilities
    z = rng.standard_normal(40)
    T, tp = 0.5, 0.7
    p = torch.softmax(torch.from_numpy(z / T), 0).numpy()
    order = np.argsort(-p)
    k = int(np.searchsorted(np.cumsum(p[order]), tp, side="left")) + 1
    nucleus = set(order[:k].tolist())
    us = (np.arange(20000) + 0.5) / 20000
    toks = np.array([O.op_sample(z, T, tp, float(u))[0] for u in us])
    assert set(toks.tolist()) == nucleus
    mass = sum(p[i] for i in nucleus)
    for i in nucleus:
        assert abs((toks == i).mean() - p[i] / mass) < 2e-4


def test_argmax_lowest_index_on_ties():
    # greedy head: the lowest index attaining the maximum.  With identical vocabulary rows every logit ties.
    w = S.make_weights(SMALL, seed=31)
    w["tok_emb"] = np.tile(w["tok_emb"][5:6], (SMALL.V, 1))
    tok = S.make_prompts(2, 3, SMALL.V, 32)
    dec = O.Decoder(SMALL, w, 2, 3)
    for i in range(3):
        lg, am = dec.column(i, tok[:, i], list(range(SMALL.L)))
        assert (lg == lg[:, :1]).all()
        assert am.tolist() == [0, 0]
    dec.close()
    # and a tie between two entries only, one of them the maximum
    w = S.make_weights(SMALL, seed=33)
    dec = O.Decoder(SMALL, w, 1, 1)
    lg, am = dec.column(0, [4], list(range(SMALL.L)))
    dec.close()
    top = int(lg[0].argmax())
    other = (top + 11) % SMALL.V
    w["tok_emb"][other] = w["tok_emb"][top]
    dec = O.Decoder(SMALL, w, 1, 1)
    lg2, am2 = dec.column(0, [4], list(range(SMALL.L)))
    dec.close()
    if 4 not in (top, other):                    # the input embedding itself was not touched
        assert lg2[0, other] == lg2[0, top] == lg2[0].max()
        assert am2[0] == min(top, other)
