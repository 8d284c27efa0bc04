"""Shared helpers for the GPU parity tests: build the same seeded model for the oracle (CPU)
and the HIP library (device), pick routers with a decision margin, compare logits."""
import torch

from oracle import first_oracle as O
from synth import CONFIGS, make_prompt, make_router, make_weights
from synth.generators import to_device

# tolerances on logits (bf16: the bar named for this build; fp32: from fp32 accumulation)
TOL = {"bf16": dict(max_abs=2e-2, rel=1e-2), "fp32": dict(max_abs=2e-4, rel=1e-4)}


def build(model, seed, max_batch=1, max_seq_len=256, router=None, page=16, desc=None, kv_layer_slots=0):
    import paper_2410_12513_amd as P
    desc = desc or CONFIGS[model]
    w = make_weights(desc, seed)
    r = make_router(desc, seed) if router is None else router
    wg = to_device(w, "cuda")
    rg = r.to("cuda").contiguous()
    ctx = P.FirstContext(desc, wg, rg, max_batch=max_batch, max_seq_len=max_seq_len, kv_page_tokens=page,
                         kv_layer_slots=kv_layer_slots)
    return desc, w, r, ctx


def routers_with_margin(desc, w, prompts, seed, tau_first=2e-5, tau=2e-3, max_tries=200, want=None):
    """Router weights drawn layer by layer from the seeded generator, re-drawn until every
    prompt's oracle rho is at least tau away from the 0.5 threshold (the paper's trained
    routers separate cleanly; random ones sit near 0.5).  Uses the oracle only.
    want: optional [prompt][layer] decisions (1 keep, 0 skip, None either) the draw must also give."""
    taps = [O.prefill_route(desc, w, torch.zeros(desc.n_layers, desc.d_model), p,
                            keep_router_inputs=True).router_in for p in prompts]
    rows = []
    for i in range(desc.n_layers):
        need = tau_first if i == 0 else tau
        for t in range(max_tries):
            cand = make_router(desc, seed * 1000 + t)[i]
            rho = [float(O.router_score(tp[i], cand.to(torch.float64))) for tp in taps]
            fits = want is None or all(want[p][i] is None or int(r >= 0.5) == int(want[p][i]) for p, r in enumerate(rho))
            if fits and all(abs(r - 0.5) >= need for r in rho):
                rows.append(cand)
                break
        else:
            raise RuntimeError(f"no router with margin for layer {i}")
    return torch.stack(rows)


def logits_close(got: torch.Tensor, ref: torch.Tensor, dtype: str):
    got = got.detach().cpu().double()
    ref = ref.detach().cpu().double()
    max_abs = float((got - ref).abs().max())
    rel = float((got - ref).norm() / ref.norm())
    ok = max_abs <= TOL[dtype]["max_abs"] and rel <= TOL[dtype]["rel"]
    return ok, max_abs, rel


def top2_gap(logits: torch.Tensor) -> float:
    v = torch.topk(logits.double(), 2).values
    return float(v[0] - v[1])
