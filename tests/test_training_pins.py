"""CPU pins of the training-side oracle (oracle/training_forward.py): soft-skip forward, loss
terms, LoRA merge.  Each pin is something the paper or the mathematics fixes, not the oracle's
own formula retyped."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import first_oracle as O
from oracle import training_forward as TF
from synth import CONFIGS, make_prompt, make_router, make_weights

F64 = torch.float64
GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "training_worked_examples.txt")) as fh:
    for line in fh:
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            GOLD[k] = [float(x) for x in v]


def _hard_forward(desc, w, ids, gates):
    """Eq. 2 on a whole sequence: H_i = H_{i-1} + g_i phi_i(H_{i-1}), g_i in {0, 1}; returns the streams entering each layer too."""
    pos = torch.arange(ids.numel())
    H = w["embed"][ids.long()].to(F64)
    taps = []
    for i, g in enumerate(gates):
        taps.append(H)
        if g:
            H, _, _ = O.block(desc, w["layers"][i], H, pos, None, None, F64)
    return H, taps


def _saturating_router(desc, w, ids, gates):
    """Router rows whose logit is exactly +-1000 on every token of the stream that reaches them (minimum-norm
    solution of H r = 1), so that sigmoid gives exactly 1.0 or 0.0 in fp64."""
    _, taps = _hard_forward(desc, w, ids, gates)
    rows = []
    for g, H in zip(gates, taps):
        r = torch.linalg.pinv(H) @ torch.ones(H.shape[0], dtype=F64)
        rows.append((1000.0 if g else -1000.0) * r)
    return torch.stack(rows)


@pytest.mark.parametrize("gates", [[1, 1, 1, 1], [1, 0, 1, 0], [0, 0, 0, 0], [0, 1, 1, 0]])
def test_saturated_routers_turn_the_soft_pass_into_the_hard_gated_pass(gates):
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 91)
    ids = make_prompt(desc.vocab, 17, 91)
    router = _saturating_router(desc, w, ids, gates)
    H, rho = TF.soft_forward(desc, w, router, ids)
    assert rho.tolist() == [float(g) for g in gates]                       # exactly 1.0 / 0.0
    ref, _ = _hard_forward(desc, w, ids, gates)
    assert float((H - ref).abs().max()) <= 1e-12 * float(ref.abs().max())
    if not any(gates):
        assert torch.equal(H, w["embed"][ids.long()].to(F64))               # nothing ran: the embedded prompt


def test_zero_router_gives_the_midpoint_of_stream_and_layer_output():
    """sigmoid(0) = 1/2 exactly: with probability 1/2 through the layer, 1/2 around it."""
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 92)
    ids = make_prompt(desc.vocab, 13, 92)
    H, rho = TF.soft_forward(desc, w, torch.zeros(desc.n_layers, desc.d_model), ids)
    assert rho.tolist() == [0.5] * desc.n_layers
    pos = torch.arange(13)
    X = w["embed"][ids.long()].to(F64)
    for i in range(desc.n_layers):
        through, _, _ = O.block(desc, w["layers"][i], X, pos, None, None, F64)
        X = 0.5 * through + 0.5 * X
    assert float((H - X).abs().max()) <= 1e-12 * float(X.abs().max())


def test_soft_pass_is_between_skipping_and_running_a_single_layer():
    """One layer, rho anywhere in (0, 1): H_1 - H_0 is rho times the layer's own update, entry by entry."""
    desc = CONFIGS["mini_bf16"].with_(n_layers=1)
    w = make_weights(desc, 93)
    ids = make_prompt(desc.vocab, 11, 93)
    router = make_router(desc, 93, std=2.0)
    H, rho = TF.soft_forward(desc, w, router, ids)
    H0 = w["embed"][ids.long()].to(F64)
    full, _ = _hard_forward(desc, w, ids, [1])
    assert 0.0 < float(rho[0]) < 1.0
    assert float(rho[0]) == float(O.router_score(H0, router[0].to(F64)))
    ratio = (H - H0) / (full - H0)
    assert float((ratio - rho[0]).abs().max()) <= 1e-9


def test_cross_entropy_against_the_library_and_closed_forms():
    rng = np.random.Generator(np.random.PCG64(94))
    logits = torch.from_numpy(rng.normal(0, 3, size=(9, 37)))
    targets = torch.tensor([3, -1, 0, 36, 5, -1, 7, 7, 1])
    ours = TF.cross_entropy(logits, targets)
    lib = F.cross_entropy(logits, targets, ignore_index=-1, reduction="mean")
    assert abs(float(ours) - float(lib)) <= 1e-12
    # hand-worked position
    row = torch.tensor([[0.0, math.log(2.0), math.log(5.0)]], dtype=F64)
    assert abs(float(TF.cross_entropy(row, torch.tensor([1]))) - GOLD["ce_example"][0]) <= 1e-15
    assert abs(GOLD["ce_example"][0] - math.log(4.0)) <= 1e-15
    # a zero head predicts the uniform distribution: ln V whatever the stream is
    desc = CONFIGS["mini_bf16"]
    w = dict(make_weights(desc, 94))
    w["lm_head"] = torch.zeros_like(w["lm_head"])
    ids = make_prompt(desc.vocab, 8, 94)
    t = TF.loss_terms(desc, w, make_router(desc, 94), ids, torch.roll(ids, -1), 0.0, 0.0)
    assert abs(float(t["ce"]) - math.log(desc.vocab)) <= 1e-12
    # no target anywhere: the term is zero, not a division by zero
    assert float(TF.cross_entropy(logits, torch.full((9,), -1))) == 0.0


def test_loss_terms_by_hand():
    R = torch.tensor([[3.0, 4.0], [0.0, 0.0], [1.0, -2.0]])
    assert float(TF.regularization(R)) == GOLD["reg_example"][0]
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 95)
    ids = make_prompt(desc.vocab, 10, 95)
    tg = torch.roll(ids, -1)
    tg[-1] = -1
    zero = torch.zeros(desc.n_layers, desc.d_model)
    t0 = TF.loss_terms(desc, w, zero, ids, tg, 0.01, 0.1)
    assert float(t0["reg"]) == 0.0 and float(t0["pp"]) == desc.n_layers / 2      # every rho is exactly 1/2
    assert float(t0["total"]) == float(t0["ce"]) + 0.1 * desc.n_layers / 2
    ones = torch.ones(desc.n_layers, desc.d_model)
    assert float(TF.regularization(ones)) == desc.n_layers * desc.d_model
    # the combination, with the worked numbers: 2 + 0.01 * 30 + 0.1 * 1.75
    assert abs(2.0 + 0.01 * GOLD["reg_example"][0] + 0.1 * GOLD["pp_example"][0] - GOLD["total_example"][0]) <= 1e-15
    router = make_router(desc, 95, std=1.0)
    t = TF.loss_terms(desc, w, router, ids, tg, 0.01, 0.1)
    assert abs(float(t["total"]) - (float(t["ce"]) + 0.01 * float((router.double() ** 2).sum()) + 0.1 * float(t["rho"].sum()))) <= 1e-12
    assert abs(float(t["pp"]) - sum(float(O.router_score(h, router[i].double())) for i, h in enumerate(_soft_taps(desc, w, router, ids)))) <= 1e-12
    # lambda and alpha enter linearly
    t2 = TF.loss_terms(desc, w, router, ids, tg, 0.03, 0.4)
    assert abs((float(t2["total"]) - float(t["total"])) - (0.02 * float(t["reg"]) + 0.3 * float(t["pp"]))) <= 1e-12


def _soft_taps(desc, w, router, ids):
    """Streams entering each layer of the soft pass, rebuilt with the midpoint form of the update."""
    pos = torch.arange(ids.numel())
    H = w["embed"][ids.long()].to(F64)
    taps = []
    for i in range(desc.n_layers):
        taps.append(H)
        rho = O.router_score(H, router[i].to(F64))
        through, _, _ = O.block(desc, w["layers"][i], H, pos, None, None, F64)
        H = rho * through + (1.0 - rho) * H
    return taps


def test_lora_merge_by_hand_and_against_the_two_branch_forward():
    W = torch.tensor([[1.0, 2.0], [3.0, 4.0]], dtype=F64)
    B = torch.tensor([[1.0], [2.0]], dtype=F64)
    A = torch.tensor([[10.0, 20.0]], dtype=F64)
    # alpha / r = 0.5 with a rank-1 pair padded to r = 2 by a zero column / row
    B2 = torch.cat([B, torch.zeros(2, 1, dtype=F64)], dim=1)
    A2 = torch.cat([A, torch.zeros(1, 2, dtype=F64)], dim=0)
    assert TF.lora_merge(W, A2, B2, 1.0, 2).flatten().tolist() == GOLD["lora_example"]
    assert 32 / 8 == GOLD["lora_paper_scale"][0]
    rng = np.random.Generator(np.random.PCG64(96))
    n, k, r = 24, 40, 8
    W = torch.from_numpy(rng.normal(0, 0.05, size=(n, k)))
    A = torch.from_numpy(rng.normal(0, 0.05, size=(r, k)))
    B = torch.from_numpy(rng.normal(0, 0.05, size=(n, r)))
    x = torch.from_numpy(rng.normal(0, 1, size=(k,)))
    merged = TF.lora_merge(W, A, B, 32.0, r)
    two_branch = W @ x + 4.0 * (B @ (A @ x))                                 # adapter beside the frozen matrix
    assert float((merged @ x - two_branch).abs().max()) <= 1e-13
    assert torch.equal(TF.lora_merge(W, A, torch.zeros_like(B), 32.0, r), W)   # B starts at zero: nothing changes
    # bf16 storage: one rounding of the exact sum
    Wb = W.to(torch.bfloat16)
    mb = TF.lora_merge(Wb, A, B, 32.0, r)
    assert mb.dtype == torch.bfloat16
    assert torch.equal(mb, (Wb.double() + 4.0 * (B @ A)).to(torch.bfloat16))
    assert not torch.equal(mb, (Wb + (4.0 * (B @ A)).to(torch.bfloat16)))    # not two roundings


def _scaled_weights(desc, seed, scale=6.0):
    """Synthetic weights blown up so that logits and the cross entropy move well away from 0 / ln V, with norm gains
    that are not all one (a dropped or misplaced gain must show)."""
    w = make_weights(desc, seed)
    g = torch.Generator().manual_seed(seed)
    w["lm_head"] = (w["lm_head"].float() * scale).to(w["lm_head"].dtype)
    w["final_norm"] = 0.5 + torch.rand(desc.d_model, generator=g)
    return w


def test_all_position_logits_against_the_pinned_single_row_head_and_a_library_twin():
    """all_position_logits is what the cross entropy sees.  Two things it shares no code with: the main oracle's
    lm_logits (pinned by the all-skip closed form), row by row on the same hidden states; and the library's
    rms_norm + linear on weights whose final-norm gains differ from one and whose head is large enough that a
    missing norm, a missing gain or a transposed head changes every logit by far more than the bar."""
    desc = CONFIGS["mini_bf16"]
    w = _scaled_weights(desc, 93)
    g = torch.Generator().manual_seed(5)
    H = torch.randn(7, desc.d_model, generator=g, dtype=F64) * 3.0
    got = TF.all_position_logits(desc, w, H)
    assert got.shape == (7, desc.vocab)
    for j in range(7):
        row = O.lm_logits(desc, w, H[j], F64).to(F64)                      # (returned as fp32)
        assert float((got[j] - row).abs().max()) <= 1e-5 * float(row.abs().max())
    twin = F.linear(F.rms_norm(H, (desc.d_model,), w["final_norm"].to(F64), desc.rms_eps), w["lm_head"].to(F64))
    assert float((got - twin).abs().max()) <= 1e-12 * float(twin.abs().max())
    assert float(got.abs().max()) > 1.0                                      # not vacuous
    # the mistakes the pin is there for are far outside the bar
    no_norm = H @ w["lm_head"].to(F64).T
    no_gain = F.linear(F.rms_norm(H, (desc.d_model,), None, desc.rms_eps), w["lm_head"].to(F64))
    assert float((got - no_norm).abs().max()) > 1e-2 and float((got - no_gain).abs().max()) > 1e-2
    # scale invariance of RMSNorm: the logits do not move when the stream is scaled (up to eps)
    big = TF.all_position_logits(desc, w, H * 64.0)
    assert float((big - got).abs().max()) <= 1e-4 * float(got.abs().max())


def test_cross_entropy_of_the_soft_pass_departs_from_ln_v_and_matches_the_library():
    """With a scaled head the loss is nowhere near ln V, so agreement with the library's cross entropy on the
    oracle's own logits (and position by position) says something about those logits."""
    desc = CONFIGS["mini_bf16"]
    w = _scaled_weights(desc, 94, scale=12.0)
    router = make_router(desc, 94)
    ids = make_prompt(desc.vocab, 11, 94)
    targets = make_prompt(desc.vocab, 11, 95).long()
    targets[3] = -1
    out = TF.loss_terms(desc, w, router, ids, targets, 0.01, 0.1)
    lg = TF.all_position_logits(desc, w, out["hidden"])
    lib = F.cross_entropy(lg, targets, ignore_index=-1, reduction="mean")
    assert abs(float(out["ce"]) - float(lib)) <= 1e-10 * abs(float(lib))
    assert abs(float(out["ce"]) - math.log(desc.vocab)) > 0.05                # the head is visible in the loss
    per_pos = F.cross_entropy(lg, targets, ignore_index=-1, reduction="none")
    keep = targets >= 0
    assert abs(float(per_pos[keep].mean()) - float(out["ce"])) <= 1e-10
