"""Temperature + top-k sampling (first_sample_top_k) against the sampling oracle, through the C ABI.
The decision is taken in fp32 on both sides; draws closer to a boundary of the cumulative
distribution than fp32 rounding can resolve may legitimately fall to either neighbour and are
checked for that instead."""
import numpy as np
import pytest
import torch

from oracle import first_oracle as O
from oracle import sampling as S
from synth import CONFIGS, make_prompt
from tests.gpu_util import build
from tests.test_gpu_path import _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)


def _ctx(model="mini_bf16", B=1, n_prompt=12, seed=71):
    desc, w, router, ctx = build(model, seed, max_seq_len=64, max_batch=B)
    prompts = [make_prompt(desc.vocab, n_prompt + b, seed + b) for b in range(B)]
    _prefill(ctx, desc, prompts)
    return desc, w, router, ctx, prompts


def _check(logits, u, T, k, got_tok, got_cand):
    """One sequence: candidates exact; token exact unless u sits on a boundary."""
    lg = logits.astype(np.float32)
    cand = S.top_k_candidates(lg, k)
    assert [int(x) for x in got_cand[:len(cand)]] == cand
    assert all(int(x) == -1 for x in got_cand[len(cand):])
    want = S.sample_top_k(lg, float(u), T, k, np.float32)
    if S.decision_margin(lg, float(u), T, k) > 1e-5:
        assert int(got_tok) == want
        return 1
    w, total = S.candidate_probabilities(lg, cand, T, np.float32)
    j = cand.index(want)
    assert int(got_tok) in cand[max(0, j - 1):j + 2]
    return 0


@pytest.mark.parametrize("V,k,T", [(1000, 10, 0.8), (2048, 1, 0.8), (2049, 10, 0.2), (5000, 64, 1.5), (37, 10, 0.8),
                                   (128256, 10, 0.8)])
def test_sampling_matches_oracle_on_synthetic_logits(V, k, T):
    import paper_2410_12513_amd as P
    from synth import ModelDesc, make_router, make_weights
    from synth.generators import to_device
    # a small model whose only relevant property is its vocabulary size
    desc = ModelDesc(n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=64, d_ffn=64, vocab=V, dtype="bf16")
    B = 3
    ctx = P.FirstContext(desc, to_device(make_weights(desc, 3), "cuda"), make_router(desc, 3).cuda(), max_batch=B, max_seq_len=32)
    ids = torch.cat([make_prompt(V, 5, 70 + b) for b in range(B)]).cuda()
    ctx.prefill_route(ids, [5] * B)
    rng = np.random.default_rng(V + k)
    exact = 0
    for trial in range(6):
        lg = (rng.normal(size=(B, V)) * rng.uniform(0.5, 5.0)).astype(np.float32)
        if trial == 1:
            lg[:, ::7] = lg[:, :1]                       # many equal logits: the index order decides
        if trial == 2:
            lg[0, :] = -1.0e30                           # all equal
            lg[1, V - 1] = 50.0                          # a single dominant token at the end of the last chunk
        u = rng.random(B).astype(np.float32)
        if trial == 3:
            u[:] = [0.0, np.float32(1.0) - np.float32(2.0 ** -24), 0.5]
        tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        cand = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
        ctx.sample_top_k(torch.from_numpy(lg).cuda(), torch.from_numpy(u).cuda(), T, k, tok, cand)
        ctx.sync()
        for b in range(B):
            exact += _check(lg[b], u[b], T, k, tok[b].item(), cand[b].cpu().numpy())
    assert exact >= 14
    ctx.close()


def test_sampled_generation_follows_the_oracle():
    """Free-running generation with sampling on the model's own logits: each step's draw is checked
    against the oracle's sampler on the library's logits, and the library's logits against the
    oracle model fed the same sampled tokens."""
    desc, w, router, ctx, prompts = _ctx("mini_bf16", B=1, n_prompt=20)
    st = O.prefill_route(desc, w, router, prompts[0])
    lg = torch.zeros(1, desc.vocab, device="cuda")
    tok = torch.zeros(1, dtype=torch.int32, device="cuda")
    cand = torch.zeros(1, 10, dtype=torch.int32, device="cuda")
    # first token: sampled from the prefill logits
    ids = prompts[0].cuda()
    ctx.prefill_route(ids, [len(prompts[0])], logits=lg)
    rng = np.random.default_rng(77)
    exact = 0
    for step in range(12):
        u = torch.tensor([rng.random()], dtype=torch.float32)
        ctx.sample_top_k(lg, u.cuda(), 0.8, 10, tok, cand)
        ctx.sync()
        exact += _check(lg[0].cpu().numpy(), float(u[0]), 0.8, 10, tok[0].item(), cand[0].cpu().numpy())
        t = int(tok[0])
        ref, _ = O.decode_step(desc, w, st, t)
        ctx.decode_step(tok, lg, tok.clone())
        ctx.sync()
        assert float((lg[0].cpu().double() - ref.double()).abs().max()) <= 2e-2
    assert exact >= 10
    ctx.close()


def test_sampling_rejects_bad_arguments():
    import paper_2410_12513_amd as P
    desc, w, router, ctx, _ = _ctx()
    lg = torch.zeros(1, desc.vocab, device="cuda")
    u = torch.zeros(1, device="cuda")
    tok = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    for T, k in ((0.0, 10), (-1.0, 10), (float("nan"), 10), (0.8, 0), (0.8, 65)):
        with pytest.raises(P.FirstError) as e:
            ctx.sample_top_k(lg, u, T, k, tok)
        assert e.value.code == -1
    ctx.sync()
    assert int(tok[0]) == -7                             # nothing written on error
    ctx.close()


@pytest.mark.parametrize("model,k", [("step_hd128", 10), ("step_hd128", 1), ("step_hd128", 15), ("step_hd128", 40),
                                     ("step_hd64", 10), ("step_3k", 7)])
def test_sampled_step_of_the_persistent_kernel_equals_step_then_sampler(model, k):
    """first_decode_step_sampled on the persistent kernel (the rule inside the kernel's LM-head epilogue; k = 40 does
    not fit its LDS and goes through the sampling kernels) against first_decode_step + first_sample_top_k in a twin
    context: logits, candidates and tokens bit-identical over free-running steps, and the draw against the oracle."""
    T = 0.8
    twins = []
    for _ in range(2):
        desc, w, router, ctx = build(model, 73, max_seq_len=96, max_batch=1)
        ctx.set_option(3, 1)                              # the persistent kernel or an error
        prompt = make_prompt(desc.vocab, 21, 73)
        lg = torch.zeros(1, desc.vocab, device="cuda")
        tok = torch.zeros(1, dtype=torch.int32, device="cuda")
        ctx.prefill_route(prompt.cuda(), [len(prompt)], logits=lg, token=tok)
        twins.append((ctx, lg, tok))
    (ca, lga, toka), (cb, lgb, tokb) = twins
    canda = torch.full((1, k), -5, dtype=torch.int32, device="cuda")
    candb = torch.full((1, k), -5, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(5)
    exact = 0
    for step in range(14):
        u = torch.tensor([rng.random()], dtype=torch.float32).cuda()
        with_logits = step % 3 != 2                        # every third step writes no logits on the fused side
        ca.decode_step_sampled(toka, u, T, k, lga if with_logits else None, toka, canda)
        cb.decode_step(tokb, lgb, tokb)
        cb.sample_top_k(lgb, u, T, k, tokb, candb)
        ca.sync(); cb.sync()
        if with_logits:
            assert torch.equal(lga, lgb)
        assert torch.equal(canda, candb), step
        assert int(toka[0]) == int(tokb[0]), step
        exact += _check(lgb[0].cpu().numpy(), float(u[0]), T, k, toka[0].item(), canda[0].cpu().numpy())
    assert exact >= 12
    assert ca.seq_len(0) == cb.seq_len(0) == 21 + 14
    ca.close(); cb.close()


def test_sampled_step_on_the_other_paths_and_its_refusals():
    """Two live sequences (no persistent kernel): the sampled step equals step + sampler; bad arguments are refused and
    change nothing."""
    import paper_2410_12513_amd as P
    twins = []
    for _ in range(2):
        desc, w, router, ctx, prompts = _ctx("mini_bf16", B=2, n_prompt=14, seed=79)
        lg = torch.zeros(2, desc.vocab, device="cuda")
        tok = torch.zeros(2, dtype=torch.int32, device="cuda")
        ids = torch.cat([p for p in prompts]).cuda()
        ctx.prefill_route(ids, [len(p) for p in prompts], logits=lg, token=tok)
        twins.append((ctx, lg, tok))
    (ca, lga, toka), (cb, lgb, tokb) = twins
    canda = torch.zeros(2, 10, dtype=torch.int32, device="cuda"); candb = torch.zeros_like(canda)
    rng = np.random.default_rng(9)
    for step in range(6):
        u = torch.tensor(rng.random(2), dtype=torch.float32).cuda()
        ca.decode_step_sampled(toka, u, 0.8, 10, lga if step % 2 == 0 else None, toka, canda)
        cb.decode_step(tokb, lgb, tokb)
        cb.sample_top_k(lgb, u, 0.8, 10, tokb, candb)
        ca.sync(); cb.sync()
        assert torch.equal(canda, candb) and torch.equal(toka, tokb)
    before = ca.seq_len(0)
    u = torch.zeros(2, device="cuda")
    for T, k in ((0.0, 10), (float("nan"), 10), (0.8, 0), (0.8, 65)):
        with pytest.raises(P.FirstError) as e:
            ca.decode_step_sampled(toka, u, T, k, lga, toka)
        assert e.value.code == -1
    assert ca.seq_len(0) == before
    ca.close(); cb.close()
