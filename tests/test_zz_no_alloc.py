"""The entry point that allocates nothing (first_sample_top_k_static: per-chunk candidate lists in a device array
that is part of the library image) against the entry point it is a variant of (first_sample_top_k, whose candidate
lists live in the context's workspace), through the C ABI: candidates and tokens bit-identical on two calls in a
row, the second with a smaller input, so that what the first call left in the shared array cannot leak into it."""
import numpy as np
import pytest
import torch

from synth import ModelDesc, make_prompt, make_router, make_weights
from synth.generators import to_device

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)


def _context(V, B):
    import paper_2410_12513_amd as P
    desc = ModelDesc(n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=64, d_ffn=64, vocab=V, dtype="bf16")
    ctx = P.FirstContext(desc, to_device(make_weights(desc, 3), "cuda"), make_router(desc, 3).cuda(), max_batch=B, max_seq_len=32)
    ids = torch.cat([make_prompt(V, 5, 70 + b) for b in range(B)]).cuda()
    ctx.prefill_route(ids, [5] * B)
    return ctx


def _both(ctx, lg, u, T, k):
    import paper_2410_12513_amd as P
    B = lg.shape[0]
    out = []
    for static in (False, True):
        tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        cand = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
        if static:
            P.sample_top_k_static(lg, u, T, k, tok, cand)
            torch.cuda.synchronize()
        else:
            ctx.sample_top_k(lg, u, T, k, tok, cand)
            ctx.sync()
        out.append((tok.cpu(), cand.cpu()))
    return out


def test_static_scratch_sampling_equals_the_context_entry_point_twice_in_a_row():
    rng = np.random.default_rng(5)
    # first call: 3 sequences, 128 256 logits each (63 chunks, ragged last one), k = 10
    big = _context(128256, 3)
    lg = torch.from_numpy((rng.normal(size=(3, 128256)) * 3.0).astype(np.float32)).cuda()
    lg[1, ::5] = lg[1, 0]                                # masses of equal logits: the index order decides
    u = torch.tensor([0.0, 0.37, 0.999], dtype=torch.float32, device="cuda")
    (t0, c0), (t1, c1) = _both(big, lg, u, 0.8, 10)
    assert torch.equal(c0, c1) and torch.equal(t0, t1)
    assert int(c0.min()) >= 0
    big.close()
    # second call, smaller in every dimension: 2 sequences, 5000 logits (3 chunks), k = 4 - the array still
    # holds the first call's lists beyond what this call writes
    small = _context(5000, 2)
    lg2 = torch.from_numpy((rng.normal(size=(2, 5000)) * 2.0).astype(np.float32)).cuda()
    u2 = torch.tensor([0.5, 0.9], dtype=torch.float32, device="cuda")
    (t0, c0), (t1, c1) = _both(small, lg2, u2, 0.8, 4)
    assert torch.equal(c0, c1) and torch.equal(t0, t1)
    # and against a plain sort of the logits (stable: equal logits by index), which is what "top k" means
    for b in range(2):
        order = np.argsort(-lg2[b].cpu().numpy(), kind="stable")[:4]
        assert [int(x) for x in c1[b]] == [int(x) for x in order]
    small.close()


def test_static_scratch_sampling_refuses_what_does_not_fit():
    import paper_2410_12513_amd as P
    lg = torch.zeros(4, 4096, device="cuda")
    u = torch.zeros(4, device="cuda")
    tok = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    for T, k in ((0.0, 10), (0.8, 0), (0.8, 65)):
        with pytest.raises(P.FirstError) as e:
            P.sample_top_k_static(lg, u, T, k, tok)
        assert e.value.code == -1
    # 1100 sequences x 2 chunks x 64 candidates = 140 800 > 131 072
    many = torch.zeros(1100, 4096, device="cuda")
    with pytest.raises(P.FirstError) as e:
        P.sample_top_k_static(many, torch.zeros(1100, device="cuda"), 0.8, 64, torch.zeros(1100, dtype=torch.int32, device="cuda"))
    assert e.value.code == -3
    torch.cuda.synchronize()
    assert int(tok[0]) == -7                             # nothing written on error
