"""CPU oracle for the training-side forward pieces of the method: the soft-skip forward pass
used while the routers are trained, the three loss terms, and the LoRA merge that makes the
fine-tuned adapters free at inference.  TEST INFRASTRUCTURE ONLY (same rules as
first_oracle.py: the HIP library never imports it and shares no code with it).  Forward
values only: no gradients, no optimiser.

What the paper fixes, and the readings taken where it is silent:

  * Soft skip (Section 4.1, last sentence of the router description, and the caption of its
    training figure: a sequence goes through layer i with probability rho_i and around it with
    probability 1 - rho_i).  The formula itself is only in the figure; the reading taken is
    the expectation of that choice,
        H_i = rho_i * (H_{i-1} + phi_i(H_{i-1})) + (1 - rho_i) * H_{i-1}
            = H_{i-1} + rho_i * phi_i(H_{i-1}),
    which becomes Eq. 2 of Section 3 when rho_i is rounded.  rho_i is the router's score of
    the stream entering layer i (the soft stream, since that is what reaches the router during
    training), one value per sequence.
  * Losses (Section 4.1): L_Reg = sum_i ||R_i||^2 over the router weight vectors, L_PP =
    sum_i rho_i, total = L_CE + lambda * L_Reg + alpha * L_PP.  L_CE is next-token cross
    entropy; the paper writes it as a sum over the data, the reading taken is the usual mean
    over the positions of a sequence that have a target (target -1 = no target), natural log.
  * LoRA (Section 4.2 and the appendix on the training set-up: rank 8, lora_alpha 32, merged
    for inference so the adapters cost no latency).  No formula is printed; the reading is the
    standard one, W' = W + (lora_alpha / r) * B A with B [out, r], A [r, in], the sum formed
    in high precision and rounded once to the storage type of W.

Pins (tests/test_training_pins.py): routers that saturate to exactly 1.0 / 0.0 turn the soft
pass into the hard-gated pass of Eq. 2 (built from the pinned layer function); the zero router
gives the midpoint of stream and layer output; cross entropy against the library routine and
the closed form ln V for a zero head; hand-worked values for L_Reg, L_PP, the total and a
2 x 2 rank-1 merge; the merged matrix applied to a vector equals the two-branch LoRA forward;
all_position_logits row by row against the main oracle's lm_logits (itself pinned by the
all-skip closed form) and against the library's rms_norm + linear on a head and gains chosen so
that a dropped norm, a dropped gain or a transposed head misses by orders of magnitude; the
cross entropy of a soft pass with a scaled head (far from ln V) against the library routine.
"""
from __future__ import annotations

import torch

from oracle import first_oracle as O


def soft_forward(desc, weights, router: torch.Tensor, ids: torch.Tensor, cdt=torch.float64):
    """Soft-skip pass over one sequence.  Returns (H_L [n, D], rho [L]) in the compute type."""
    n = int(ids.numel())
    pos = torch.arange(n)
    H = weights["embed"][ids.long()].to(cdt)
    rhos = []
    for i in range(desc.n_layers):
        rho = O.router_score(H, router[i].to(cdt))
        through, _, _ = O.block(desc, weights["layers"][i], H, pos, None, None, cdt)   # H + phi_i(H)
        H = H + rho * (through - H)
        rhos.append(rho)
    return H, torch.stack(rhos)


def all_position_logits(desc, weights, H: torch.Tensor, cdt=torch.float64) -> torch.Tensor:
    """W_lm . RMSNorm(H[j]; g_final) for every position j: [n, V]."""
    x = O.rmsnorm(H, weights["final_norm"].to(cdt), desc.rms_eps)
    return x @ weights["lm_head"].to(cdt).T


def cross_entropy(logits: torch.Tensor, targets: torch.Tensor) -> torch.Tensor:
    """Mean over the positions with targets[j] >= 0 of  log(sum_v exp(l[j, v])) - l[j, targets[j]]."""
    total, count = logits.new_zeros(()), 0
    for j in range(logits.shape[0]):
        t = int(targets[j])
        if t < 0:
            continue
        row = logits[j]
        m = row.max()
        total = total + (m + torch.log(torch.exp(row - m).sum()) - row[t])
        count += 1
    return total / count if count else total


def regularization(router: torch.Tensor, cdt=torch.float64) -> torch.Tensor:
    """L_Reg = sum_i ||R_i||^2."""
    return (router.to(cdt) ** 2).sum()


def loss_terms(desc, weights, router, ids, targets, lam: float, alpha: float, cdt=torch.float64):
    """The three terms and their combination for one sequence, plus H_L and rho."""
    H, rho = soft_forward(desc, weights, router, ids, cdt)
    ce = cross_entropy(all_position_logits(desc, weights, H, cdt), targets)
    reg = regularization(router, cdt)
    pp = rho.sum()
    return dict(ce=ce, reg=reg, pp=pp, total=ce + lam * reg + alpha * pp, hidden=H, rho=rho)


def lora_merge(W: torch.Tensor, A: torch.Tensor, B: torch.Tensor, lora_alpha: float, r: int) -> torch.Tensor:
    """W + (lora_alpha / r) * B A, formed in fp64 and rounded once to W's type.  W [out, in], B [out, r], A [r, in]."""
    assert A.shape[0] == r and B.shape[1] == r
    merged = W.double() + (float(lora_alpha) / r) * (B.double() @ A.double())
    return merged.to(W.dtype)
