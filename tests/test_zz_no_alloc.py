"""skd_logits_argmax_noalloc (LM-head partials in a static device array) against skd_logits_argmax.

Two calls in a row through the C ABI, the second on a smaller problem (fewer rows, smaller vocabulary), so the
second finds the first call's partials still in the shared array; then both again after a decode step.  Outputs
must be bit-identical to the allocating entry point's (same kernels), and device memory in use must not change
across the calls.
"""
import numpy as np
import pytest

import synth_inputs as S
from paper_2307_02628_amd import skd

pytestmark = pytest.mark.gpu


def _state(torch, shape, B, P, N, seed, stream):
    w = S.weights_to_bf16_values(S.make_weights(shape, seed))
    cfg = skd.make_config(shape, B, P, N, 1, shape.L, dtype=skd.BF16, io_on_device=1)
    dec = skd.Decoder(cfg, w, stream=stream.cuda_stream)
    pr = torch.from_numpy(np.ascontiguousarray(S.make_prompts(B, P, shape.V, seed + 1).T)).cuda()   # [P][B]
    tape = torch.from_numpy(S.make_token_tape(B, N - P, shape.V, seed + 2)).cuda()
    return dec, pr, tape


def test_noalloc_argmax_matches_allocating_entry_point():
    import torch
    big = S.ModelShape(L=2, d=256, H=4, f=512, V=5003, max_pos=32)
    small = S.ModelShape(L=2, d=128, H=2, f=256, V=777, max_pos=32)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        states = [_state(torch, big, 33, 7, 12, 90, stream), _state(torch, small, 3, 5, 12, 95, stream)]
        bufs = []
        for dec, pr, _ in states:
            B, V = dec.cfg.batch, dec.cfg.vocab
            bufs.append({k: (torch.full((B,), -7, dtype=torch.int32, device="cuda"),
                             torch.full((B, V), float("nan"), dtype=torch.float32, device="cuda")) for k in ("ref", "new")})
            dec.prefill(pr)
        torch.cuda.synchronize()
        for step in range(3):
            free0 = torch.cuda.mem_get_info()[0]
            for (dec, _, _), buf in zip(states, bufs):                       # the big problem, then the small one
                assert dec.logits_argmax_noalloc_rc(*buf["new"]) == skd.OK
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free0                     # nothing was allocated
            for (dec, _, tape), buf in zip(states, bufs):
                dec.logits_argmax_device(*buf["ref"])
                dec.synchronize()
                tok_ref, lg_ref = (x.cpu().numpy() for x in buf["ref"])
                tok_new, lg_new = (x.cpu().numpy() for x in buf["new"])
                assert np.isfinite(lg_ref).all()
                np.testing.assert_array_equal(lg_new, lg_ref)
                np.testing.assert_array_equal(tok_new, tok_ref)
                np.testing.assert_array_equal(tok_new, lg_ref.argmax(-1))
                buf["new"][0].fill_(-7)
                buf["new"][1].fill_(float("nan"))
                t = dec.cfg.prompt_size + step
                dec.decode_step(t, tape[step])
        # tokens only / logits only
        dec, _, _ = states[1]
        tok, lg = bufs[1]["new"]
        assert dec.logits_argmax_noalloc_rc(tok, None) == skd.OK
        assert dec.logits_argmax_noalloc_rc(None, lg) == skd.OK
        dec.decode_step(dec.cfg.prompt_size + 3, None)                       # continues from the tokens kept inside
        dec.synchronize()
        np.testing.assert_array_equal(tok.cpu().numpy(), lg.cpu().numpy().argmax(-1))
        for dec, _, _ in states:
            dec.close()


def test_noalloc_argmax_refusals():
    import torch
    shape = S.ModelShape(L=1, d=128, H=2, f=64, V=140000, max_pos=8)      # 2188 workgroups x 128 rows > 262144 partials
    w = S.weights_to_bf16_values(S.make_weights(shape, 97))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        cfg = skd.make_config(shape, 100, 2, 4, 1, 1, dtype=skd.BF16, io_on_device=1)
        with skd.Decoder(cfg, w, stream=stream.cuda_stream) as dec:
            tok = torch.zeros(100, dtype=torch.int32, device="cuda")
            assert dec.logits_argmax_noalloc_rc(tok, None) == skd.ERR_ORDER      # nothing processed yet
            dec.prefill(torch.from_numpy(np.ascontiguousarray(S.make_prompts(100, 2, shape.V, 98).T)).cuda())
            assert dec.logits_argmax_noalloc_rc(tok, None) == skd.ERR_RANGE      # beyond the static scratch
            dec.logits_argmax_device(tok, None)                                   # the allocating entry point still works
            dec.synchronize()
    tiny = S.TINY
    wt = S.weights_to_bf16_values(S.make_weights(tiny, 0))
    pr = S.make_prompts(2, 16, tiny.V, 1)
    with skd.Decoder(skd.make_config(tiny, 2, 16, 32, 2, 4, dtype=skd.BF16), wt) as dec:      # host I/O
        dec.prefill(pr)
        assert dec.logits_argmax_noalloc_rc(None, None) == skd.ERR_SHAPE
    with skd.Decoder(skd.make_config(tiny, 2, 16, 32, 2, 4, dtype=skd.FP32, io_on_device=1),
                     S.make_weights(tiny, 0)) as dec:                                         # fp32 debug path
        assert dec.logits_argmax_noalloc_rc(None, None) in (skd.ERR_ORDER, skd.ERR_SHAPE)
    assert skd.lib().skd_logits_argmax_noalloc(None, None, None) == skd.ERR_NULL
