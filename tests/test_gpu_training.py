"""Training-side forward pieces through the C ABI against oracle/training_forward.py: the soft-skip
forward with its loss terms (first_soft_forward) and the LoRA merge (first_lora_merge)."""
import math

import numpy as np
import pytest
import torch

import paper_2410_12513_amd as P
from oracle import first_oracle as O
from oracle import training_forward as TF
from synth import CONFIGS, make_prompt, make_router, make_weights
from synth.generators import to_device
from tests.gpu_util import TOL, build, logits_close
from tests.test_gpu_path import _decode, _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)

# |dCE| of one position <= 2 max|dlogit| (log-sum-exp and the pick are both 1-Lipschitz in the max norm)
CE_TOL = {"bf16": 2 * 2e-2, "fp32": 2 * 2e-4}


def _targets(prompt, holes=()):
    t = torch.roll(prompt, -1).to(torch.int32)
    t[-1] = -1
    for j in holes:
        t[j] = -1
    return t


def _soft(ctx, desc, prompts, targets, lam, alpha):
    B, n = len(prompts), sum(p.numel() for p in prompts)
    out = dict(terms=torch.zeros(B, 4, device="cuda"), rho=torch.zeros(B, desc.n_layers, device="cuda"),
               hidden=torch.zeros(n, desc.d_model, device="cuda"))
    ctx.soft_forward(torch.cat(prompts).to(torch.int32).cuda(), [p.numel() for p in prompts],
                     torch.cat(targets).to(torch.int32).cuda(), lam, alpha, **out)
    return {k: v.cpu() for k, v in out.items()}


@pytest.mark.parametrize("model,lens", [("mini_bf16", [70, 131]), ("mini_fp32", [53, 9]), ("step_hd128", [150]),
                                        ("mini_hd128", [1, 40])])
def test_soft_forward_and_loss_terms_match_oracle(model, lens):
    desc = CONFIGS[model]
    router = make_router(desc, 97, std=1.5)                      # scores spread over (0, 1)
    desc, w, router, ctx = build(model, 97, max_batch=len(lens), max_seq_len=max(lens) + 8, router=router)
    prompts = [make_prompt(desc.vocab, n, 97 + b) for b, n in enumerate(lens)]
    targets = [_targets(p, holes=(3,) if p.numel() > 8 else ()) for p in prompts]
    lam, alpha = 0.01, 0.05
    got = _soft(ctx, desc, prompts, targets, lam, alpha)
    off = 0
    for b, (p, t) in enumerate(zip(prompts, targets)):
        ref = TF.loss_terms(desc, w, router, p, t, lam, alpha)
        n = p.numel()
        assert float((got["rho"][b].double() - ref["rho"]).abs().max()) <= (2e-3 if desc.dtype == "bf16" else 1e-5)
        h = got["hidden"][off:off + n].double()
        assert float((h - ref["hidden"]).norm() / ref["hidden"].norm()) <= TOL[desc.dtype]["rel"]
        ce, reg, pp, total = [float(x) for x in got["terms"][b]]
        assert abs(ce - float(ref["ce"])) <= CE_TOL[desc.dtype], (ce, float(ref["ce"]))
        assert abs(reg - float(ref["reg"])) <= 1e-5 * float(ref["reg"])
        assert abs(pp - float(ref["pp"])) <= desc.n_layers * (2e-3 if desc.dtype == "bf16" else 1e-5)
        assert abs(total - (ce + lam * reg + alpha * pp)) <= 1e-5 * max(1.0, abs(total))
        assert abs(total - float(ref["total"])) <= CE_TOL[desc.dtype] + alpha * desc.n_layers * 2e-3
        off += n
    # a training pass leaves nothing to decode
    tin = torch.tensor([1] * len(lens), dtype=torch.int32, device="cuda")
    with pytest.raises(P.FirstError) as e:
        ctx.decode_step(tin, None, tin)
    assert e.value.code == -2
    ctx.close()


@pytest.mark.parametrize("model,n", [("mini_bf16", 131), ("mini_fp32", 40), ("step_hd128", 150)])
def test_cross_entropy_sees_the_lm_head(model, n):
    """With N(0, 0.02) weights the cross entropy sits within 0.1 of ln V whatever the logits are, so the bar above barely
    sees the head.  Here the head is scaled by 12 and the final-norm gains are spread over [0.5, 1.5): the loss is far
    from ln V, and it is compared with the oracle's head and cross entropy applied to the hidden states THE LIBRARY
    returned - what is left is the error of the library's own norm + head + loss, a few fp32 roundings of logits of
    size ~10 (the bf16 head weights are exact on both sides, activations enter with 16 mantissa bits) - and with the
    whole oracle pass at a bar derived from the hidden-state tolerance."""
    desc = CONFIGS[model]
    w = make_weights(desc, 99)
    g = torch.Generator().manual_seed(99)
    w["lm_head"] = (w["lm_head"].float() * 12.0).to(w["lm_head"].dtype)
    w["final_norm"] = 0.5 + torch.rand(desc.d_model, generator=g)
    router = make_router(desc, 99, std=1.5)
    ctx = P.FirstContext(desc, to_device(w, "cuda"), router.cuda(), max_batch=1, max_seq_len=n + 8)
    prompt = make_prompt(desc.vocab, n, 99)
    tg = _targets(prompt, holes=(3,))
    got = _soft(ctx, desc, [prompt], [tg], 0.0, 0.0)
    ce = float(got["terms"][0][0])
    lg_own = TF.all_position_logits(desc, w, got["hidden"].double())
    ce_own = float(TF.cross_entropy(lg_own, tg))
    assert abs(ce_own - math.log(desc.vocab)) > 0.05                       # the head is visible in the loss
    scale = float(lg_own.abs().max())
    assert abs(ce - ce_own) <= 2 * 1e-4 * scale, (ce, ce_own, scale)       # |dCE| <= 2 max|dlogit|, logits to ~1e-5 relative
    ref = TF.loss_terms(desc, w, router, prompt, tg, 0.0, 0.0)
    rel_h = float((got["hidden"].double() - ref["hidden"]).norm() / ref["hidden"].norm())
    assert rel_h <= TOL[desc.dtype]["rel"]
    # hidden states off by rel_h (L2) move a logit by at most about rel_h * sqrt(D) * |logit| in the worst case; the
    # observed effect is far smaller, so the bar is 2 * 8 * rel_h * scale
    assert abs(ce - float(ref["ce"])) <= 16 * max(rel_h, 1e-6) * scale, (ce, float(ref["ce"]), rel_h, scale)
    ctx.close()


def test_zero_router_saturated_router_and_no_targets():
    desc = CONFIGS["mini_bf16"]
    L = desc.n_layers
    w = make_weights(desc, 98)
    prompt = make_prompt(desc.vocab, 61, 98)
    tg = _targets(prompt)
    # zero router: every rho is exactly 1/2, L_Reg = 0, L_PP = L / 2
    _, _, _, ctx = build("mini_bf16", 98, max_seq_len=80, router=torch.zeros(L, desc.d_model))
    got = _soft(ctx, desc, [prompt], [tg], 0.5, 0.25)
    assert got["rho"][0].tolist() == [0.5] * L
    ce, reg, pp, total = [float(x) for x in got["terms"][0]]
    assert reg == 0.0 and pp == L / 2 and abs(total - (ce + 0.25 * L / 2)) <= 1e-6
    # no position has a target: L_CE = 0
    got = _soft(ctx, desc, [prompt], [torch.full_like(tg, -1)], 0.5, 0.25)
    assert float(got["terms"][0][0]) == 0.0 and float(got["terms"][0][3]) == 0.25 * L / 2
    ctx.close()
    # routers that give exactly 1.0 on the stream they see: the soft pass is the prompt pass of prefill
    pos = torch.arange(61)
    H = w["embed"][prompt.long()].double()
    rows = []
    for i in range(L):
        rows.append(1000.0 * (torch.linalg.pinv(H) @ torch.ones(61, dtype=torch.float64)))
        H, _, _ = O.block(desc, w["layers"][i], H, pos, None, None, torch.float64)
    router = torch.stack(rows).float()
    _, _, _, ctx = build("mini_bf16", 98, max_seq_len=80, router=router)
    got = _soft(ctx, desc, [prompt], [tg], 0.0, 1.0)
    assert got["rho"][0].tolist() == [1.0] * L and float(got["terms"][0][2]) == float(L)
    pre = _prefill(ctx, desc, [prompt])
    # p + 1.0 * (H - p) rounds differently from H: a few fp32 ulps per layer, carried through the later layers
    gap, scale = float((got["hidden"][60] - pre["hidden"][0]).abs().max()), float(pre["hidden"][0].abs().max())
    assert gap <= 1e-4 * scale, (gap, scale)
    # ... and the context decodes as usual after a training pass
    lg, _ = _decode(ctx, desc, [[int(pre["token"][0])]])
    st = O.prefill_route(desc, w, router, prompt)
    ref, _ = O.decode_step(desc, w, st, int(pre["token"][0]))
    ok, ma, rel = logits_close(lg[0, 0], ref, desc.dtype)
    assert ok, (ma, rel)
    ctx.close()


@pytest.mark.parametrize("dtype,n,k,r", [("bf16", 300, 1096, 8), ("bf16", 37, 2048, 32), ("fp32", 130, 520, 8),
                                         ("bf16", 1, 8, 1), ("bf16", 4096, 4096, 8)])
def test_lora_merge_matches_oracle(dtype, n, k, r):
    rng = np.random.Generator(np.random.PCG64(99))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    W = torch.from_numpy(rng.normal(0, 0.02, size=(n, k))).to(tdt)
    A = torch.from_numpy(rng.normal(0, 0.02, size=(r, k))).float()
    Bm = torch.from_numpy(rng.normal(0, 0.02, size=(n, r))).float()
    ref = TF.lora_merge(W, A, Bm, 4.0 * r, r)                     # scale = lora_alpha / r = 4 as in the paper's setting
    Wd = W.cuda()
    P.lora_merge(Wd, A.cuda(), Bm.cuda(), 4.0)
    torch.cuda.synchronize()
    got = Wd.cpu()
    if dtype == "bf16":
        # fp32 sum against the oracle's fp64: the rounding to bf16 may fall the other way for values within
        # fp32 error of a rounding boundary - by one step of the result, rarely; where W and the update
        # nearly cancel, the fp32 error of the operands (not of the tiny result) is the measure
        upd = 4.0 * (Bm.double() @ A.double())
        err = (got.double() - ref.double()).abs()
        allowed = ref.double().abs() * 2.0 ** -7 + 1e-6 * (W.double().abs() + upd.abs())
        assert bool((err <= allowed).all()), float((err - allowed).max())
        assert float((got != ref).float().mean()) <= 1e-3
    else:
        assert float((got.double() - ref.double()).abs().max()) <= 1e-6 * float(ref.abs().max())
    assert not torch.equal(got, W)
    # B = 0 (how LoRA starts): bit-identical
    Wd = W.cuda()
    P.lora_merge(Wd, A.cuda(), torch.zeros_like(Bm).cuda(), 4.0)
    torch.cuda.synchronize()
    assert torch.equal(Wd.cpu(), W)


def test_lora_merge_refuses_bad_shapes():
    W = torch.zeros(16, 64, dtype=torch.bfloat16, device="cuda")
    for r, k in ((33, 64), (0, 64)):
        with pytest.raises(P.FirstError) as e:
            P.lora_merge(W, torch.zeros(r, 64, device="cuda"), torch.zeros(16, r, device="cuda"), 1.0)
        assert e.value.code == -1
    W = torch.zeros(16, 60, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.FirstError):
        P.lora_merge(W, torch.zeros(8, 60, device="cuda"), torch.zeros(16, 8, device="cuda"), 1.0)


def test_merged_adapters_enter_the_path():
    """Adapters on the attention and MLP matrices of every layer (Section 4.2), merged on the device,
    then prefill + decode against the oracle run on weights merged by the oracle."""
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 101)
    rng = np.random.Generator(np.random.PCG64(101))
    wg = to_device(w, "cuda")
    wm = dict(w)
    wm["layers"] = [dict(l) for l in w["layers"]]
    r = 8
    for i in range(desc.n_layers):
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            n, k = w["layers"][i][name].shape
            A = torch.from_numpy(rng.normal(0, 0.05, size=(r, k))).float()
            Bm = torch.from_numpy(rng.normal(0, 0.05, size=(n, r))).float()
            wm["layers"][i][name] = TF.lora_merge(w["layers"][i][name], A, Bm, 32.0, r)
            P.lora_merge(wg["layers"][i][name], A.cuda(), Bm.cuda(), 32.0 / r)
    torch.cuda.synchronize()
    assert not torch.equal(wm["layers"][0]["wq"], w["layers"][0]["wq"])
    router = make_router(desc, 101)
    ctx = P.FirstContext(desc, wg, router.cuda(), max_batch=1, max_seq_len=64)
    prompt = make_prompt(desc.vocab, 37, 101)
    got = _prefill(ctx, desc, [prompt])
    st = O.prefill_route(desc, wm, router, prompt)
    ok, ma, rel = logits_close(got["logits"][0], st.logits, desc.dtype)
    assert ok, (ma, rel)
    plain = O.prefill_route(desc, w, router, prompt)
    assert float((st.logits - plain.logits).abs().max()) > 10 * ma       # the adapters matter at this size
    ctx.set_mask(0, [1, 0, 1, 1]); st.set_mask([1, 0, 1, 1])
    lg, _ = _decode(ctx, desc, [[st.token]])
    ref, _ = O.decode_step(desc, wm, st, st.token)
    ok, ma, rel = logits_close(lg[0, 0], ref, desc.dtype)
    assert ok, (ma, rel)
    ctx.close()
