"""Pins for the CPU oracle: checks against things fixed by the paper or by mathematics,
none of which re-use the oracle's own formulas.

  * recompute():   an independent no-cache forward built on library attention / norm / SiLU
                   and complex-number RoPE (Section 2 Eq. 1; Section 4.3 items 1-2)
  * scalar twin:   pure-Python loops over a toy model (brute force)
  * closed forms:  all-skip = embedding -> final norm -> LM head; zero router -> rho = 0.5
                   exactly -> keep; router aligned with the stream -> rho -> 1 / 0
  * invariants:    prefill independent of routers; skipped layer leaves state untouched;
                   pruned-model equivalence (Section 3 Eq. 2); RoPE relative-position law
  * printed value: router parameter fractions (Section 5)
"""
import math
import os

import pytest
import torch
import torch.nn.functional as F

from oracle import first_oracle as O
from synth import CONFIGS, ModelDesc, make_prompt, make_router, make_skip_mask, make_weights

torch.set_grad_enabled(False)
F64 = torch.float64

TOY = ModelDesc(n_layers=3, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24,
                vocab=29, dtype="fp32")
SMALL = ModelDesc(n_layers=4, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=176,
                  vocab=211, dtype="fp32")


def _scaled(desc, seed, scale=8.0):
    """Weights with a larger spread than N(0,0.02) so every term matters numerically."""
    w = make_weights(desc, seed)
    for k in ("embed", "lm_head"):
        w[k] = w[k] * scale
    for lw in w["layers"]:
        for k in lw:
            if k.endswith("norm"):
                lw[k] = lw[k] + 0.1 * torch.arange(lw[k].numel(), dtype=torch.float32) / lw[k].numel()
            else:
                lw[k] = lw[k] * scale
    w["final_norm"] = w["final_norm"] + 0.05
    return w


# ----------------------------------------------------------------------------------------
# Independent recompute: library ops, no cache, whole blocks of rows at once.
def _rope_complex(x, pos, base):
    n, H, hd = x.shape
    half = hd // 2
    z = torch.complex(x[..., :half], x[..., half:])
    inv = torch.tensor([base ** (-(2.0 * d) / hd) for d in range(half)], dtype=F64)
    rot = torch.polar(torch.ones(n, half, dtype=F64), pos.to(F64)[:, None] * inv[None, :])
    z = z * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def _lib_block(desc, lw, H, pos, K_ctx, V_ctx):
    """One decoder block over rows H at positions pos; K_ctx/V_ctx are earlier keys/values
    (all visible to every row).  Returns new H and this block's own K, V (unrounded)."""
    Hq, Hkv, hd = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    n = H.shape[0]
    x = F.rms_norm(H, (desc.d_model,), lw["attn_norm"].to(F64), desc.rms_eps)
    q = _rope_complex(F.linear(x, lw["wq"].to(F64)).view(n, Hq, hd), pos, desc.rope_base)
    k = _rope_complex(F.linear(x, lw["wk"].to(F64)).view(n, Hkv, hd), pos, desc.rope_base)
    v = F.linear(x, lw["wv"].to(F64)).view(n, Hkv, hd)
    Kf = k if K_ctx is None else torch.cat([K_ctx, k])
    Vf = v if V_ctx is None else torch.cat([V_ctx, v])
    nctx = Kf.shape[0] - n
    am = torch.ones(n, Kf.shape[0], dtype=torch.bool)
    am[:, nctx:] = torch.tril(torch.ones(n, n, dtype=torch.bool))
    rep = Hq // Hkv
    a = F.scaled_dot_product_attention(q.transpose(0, 1)[None],
                                       Kf.repeat_interleave(rep, dim=1).transpose(0, 1)[None],
                                       Vf.repeat_interleave(rep, dim=1).transpose(0, 1)[None],
                                       attn_mask=am)[0].transpose(0, 1).reshape(n, Hq * hd)
    u = H + F.linear(a, lw["wo"].to(F64))
    y = F.rms_norm(u, (desc.d_model,), lw["mlp_norm"].to(F64), desc.rms_eps)
    z = F.silu(F.linear(y, lw["w_gate"].to(F64))) * F.linear(y, lw["w_up"].to(F64))
    return u + F.linear(z, lw["w_down"].to(F64)), k, v


def recompute(desc, w, prompt, gen_inputs, mask):
    """Logits for every decode input, with the method's semantics: the prompt goes through
    every layer; the decode rows go through kept layers only and see, in a kept layer,
    the prompt keys made on the full stream plus the decode keys made on the gated one."""
    n = prompt.numel()
    Hp = w["embed"][prompt.long()].to(F64)
    Hd = w["embed"][torch.as_tensor(gen_inputs).long()].to(F64)
    pos_p = torch.arange(n)
    pos_d = torch.arange(n, n + len(gen_inputs))
    for i, lw in enumerate(w["layers"]):
        Hp, kp, vp = _lib_block(desc, lw, Hp, pos_p, None, None)
        if int(mask[i]):
            Hd, _, _ = _lib_block(desc, lw, Hd, pos_d, kp, vp)
    first = F.linear(F.rms_norm(Hp[-1], (desc.d_model,), w["final_norm"].to(F64), desc.rms_eps),
                     w["lm_head"].to(F64))
    rest = F.linear(F.rms_norm(Hd, (desc.d_model,), w["final_norm"].to(F64), desc.rms_eps),
                    w["lm_head"].to(F64))
    return first, rest


@pytest.mark.parametrize("cdt", [torch.float64, torch.float32], ids=["fp64", "fp32"])
@pytest.mark.parametrize("mask_kind", ["all_keep", "interior", "all_skip", "first_only"])
def test_cached_decode_equals_independent_recompute(mask_kind, cdt):
    """Also in the oracle's fp32 mode ("full precision" arithmetic, the mode the CPU baseline is timed in): the same
    definition with fp32 accumulation must stay within fp32 rounding of the fp64 recompute."""
    desc = SMALL
    w = _scaled(desc, 11)
    router = make_router(desc, 11)
    prompt = make_prompt(desc.vocab, 13, 11)
    L = desc.n_layers
    mask = {"all_keep": [1] * L, "interior": [1, 0, 1, 1][:L], "all_skip": [0] * L,
            "first_only": [1] + [0] * (L - 1)}[mask_kind]
    st = O.prefill_route(desc, w, router, prompt, cdt=cdt)
    st.set_mask(mask)
    inputs = [st.token] + [int(t) for t in make_prompt(desc.vocab, 6, 12)]
    lg, _ = O.generate(desc, w, st, len(inputs), cdt=cdt, forced=inputs)
    first, rest = recompute(desc, w, prompt, inputs, mask)
    # fp32 KV storage against an unrounded recompute: 1e-6-level agreement expected (fp32 arithmetic: 1e-4)
    tol = 1e-5 if cdt == torch.float64 else 2e-4
    assert torch.allclose(st.logits.to(F64), first, rtol=tol, atol=tol)
    assert torch.allclose(lg.to(F64), rest, rtol=tol, atol=tol)
    assert lg.abs().max() > 0.5          # the comparison is not vacuous


def test_all_keep_free_running_equals_plain_transformer():
    """All-keep decode = the unmodified model run on prompt + generated tokens."""
    desc = SMALL
    w = _scaled(desc, 21)
    prompt = make_prompt(desc.vocab, 9, 21)
    st = O.prefill_route(desc, w, torch.zeros(desc.n_layers, desc.d_model), prompt)
    assert st.mask.tolist() == [1] * desc.n_layers
    lg, toks = O.generate(desc, w, st, 5)
    seq = torch.cat([prompt, torch.tensor([st.token] + toks[:-1], dtype=torch.int32)])
    # plain model: every row through every layer, one causal pass
    H = w["embed"][seq.long()].to(F64)
    for lw in w["layers"]:
        H, _, _ = _lib_block(desc, lw, H, torch.arange(seq.numel()), None, None)
    full = F.linear(F.rms_norm(H, (desc.d_model,), w["final_norm"].to(F64), desc.rms_eps),
                    w["lm_head"].to(F64))
    assert torch.allclose(lg.to(F64), full[prompt.numel():], rtol=1e-5, atol=1e-5)
    assert torch.allclose(st.logits.to(F64), full[prompt.numel() - 1], rtol=1e-5, atol=1e-5)


# ----------------------------------------------------------------------------------------
# Scalar pure-Python twin (brute force on a toy model).
def _twin(desc, w, router, prompt, mask, gen_inputs):
    D, Hq, Hkv, hd, Fd, V = (desc.d_model, desc.n_q_heads, desc.n_kv_heads, desc.head_dim,
                             desc.d_ffn, desc.vocab)
    tl = lambda t: t.to(F64).tolist()
    E, Wlm, gf = tl(w["embed"]), tl(w["lm_head"]), tl(w["final_norm"])
    LW = [{k: tl(v) for k, v in lw.items()} for lw in w["layers"]]
    R = tl(router)
    f32 = lambda v: float(torch.tensor(v, dtype=torch.float32))   # KV storage rounding

    def norm(x, g):
        r = math.sqrt(sum(a * a for a in x) / len(x) + desc.rms_eps)
        return [a / r * b for a, b in zip(x, g)]

    def matvec(W, x):
        return [sum(W[r][c] * x[c] for c in range(len(x))) for r in range(len(W))]

    def rot(vec, p):
        out = list(vec)
        for h in range(len(vec) // hd):
            for d in range(hd // 2):
                th = p * desc.rope_base ** (-2.0 * d / hd)
                a, b = vec[h * hd + d], vec[h * hd + d + hd // 2]
                out[h * hd + d] = a * math.cos(th) - b * math.sin(th)
                out[h * hd + d + hd // 2] = b * math.cos(th) + a * math.sin(th)
        return out

    Kc = [[] for _ in range(desc.n_layers)]
    Vc = [[] for _ in range(desc.n_layers)]

    def layer(i, h, p):
        lw = LW[i]
        x = norm(h, lw["attn_norm"])
        q = rot(matvec(lw["wq"], x), p)
        k = rot(matvec(lw["wk"], x), p)
        v = matvec(lw["wv"], x)
        Kc[i].append([f32(a) for a in k])
        Vc[i].append([f32(a) for a in v])
        att = [0.0] * (Hq * hd)
        for hh in range(Hq):
            g = hh // (Hq // Hkv)
            sc = [sum(q[hh * hd + d] * Kc[i][j][g * hd + d] for d in range(hd)) / math.sqrt(hd)
                  for j in range(p + 1)]
            mx = max(sc)
            e = [math.exp(s - mx) for s in sc]
            z = sum(e)
            for d in range(hd):
                att[hh * hd + d] = sum(e[j] / z * Vc[i][j][g * hd + d] for j in range(p + 1))
        u = [a + b for a, b in zip(h, matvec(lw["wo"], att))]
        y = norm(u, lw["mlp_norm"])
        gt, up = matvec(lw["w_gate"], y), matvec(lw["w_up"], y)
        z = [a / (1.0 + math.exp(-a)) * b for a, b in zip(gt, up)]
        return [a + b for a, b in zip(u, matvec(lw["w_down"], z))]

    n = len(prompt)
    # prompt: position by position, every layer; router sums gathered on the way
    sig_sum = [0.0] * desc.n_layers
    last = None
    for p in range(n):
        h = list(E[prompt[p]])
        for i in range(desc.n_layers):
            zdot = sum(a * b for a, b in zip(R[i], h))
            sig_sum[i] += 1.0 / (1.0 + math.exp(-zdot))
            h = layer(i, h, p)
        last = h
    rho = [s / n for s in sig_sum]
    first_logits = matvec(Wlm, norm(last, gf))
    outs = []
    for s, t in enumerate(gen_inputs):
        h = list(E[t])
        for i in range(desc.n_layers):
            if mask[i]:
                h = layer(i, h, n + s)
        outs.append(matvec(Wlm, norm(h, gf)))
    return rho, first_logits, outs


@pytest.mark.parametrize("cdt", [torch.float64, torch.float32], ids=["fp64", "fp32"])
def test_scalar_twin_on_toy_model(cdt):
    desc = TOY
    w = _scaled(desc, 5, scale=20.0)
    router = make_router(desc, 5, std=1.0)
    prompt = make_prompt(desc.vocab, 6, 5)
    mask = [1, 0, 1]
    st = O.prefill_route(desc, w, router, prompt, cdt=cdt)
    rho_o = st.rho.clone()
    st.set_mask(mask)
    inputs = [st.token, 3, 17, 8]
    lg, _ = O.generate(desc, w, st, len(inputs), cdt=cdt, forced=inputs)
    rho_t, first_t, outs_t = _twin(desc, w, router, prompt.tolist(), mask, inputs)
    tol = 1.0 if cdt == torch.float64 else 30.0             # (the fp32 mode against the fp64 scalar twin)
    assert torch.allclose(rho_o.to(F64), torch.tensor(rho_t, dtype=F64), atol=1e-6 * tol)
    assert torch.allclose(st.logits.to(F64), torch.tensor(first_t, dtype=F64), rtol=1e-5 * tol, atol=1e-6 * tol)
    assert torch.allclose(lg.to(F64), torch.tensor(outs_t, dtype=F64), rtol=1e-5 * tol, atol=1e-6 * tol)
    assert (rho_o - 0.5).abs().max() > 1e-3 and lg.abs().max() > 0.1


# ----------------------------------------------------------------------------------------
def test_all_skip_closed_form():
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 31)
    prompt = make_prompt(desc.vocab, 20, 31)
    st = O.prefill_route(desc, w, make_router(desc, 31), prompt)
    st.set_mask([0] * desc.n_layers)
    k_before = [k.clone() for k in st.K]
    tok = 77
    lg, _ = O.decode_step(desc, w, st, tok)
    e = w["embed"][tok].to(torch.float64).numpy()
    import numpy as np
    x = e / np.sqrt((e * e).mean() + desc.rms_eps) * w["final_norm"].to(F64).numpy()
    ref = w["lm_head"].to(F64).numpy() @ x
    assert np.allclose(lg.numpy(), ref.astype(np.float32), rtol=1e-6, atol=1e-7)
    assert all(torch.equal(a, b) for a, b in zip(k_before, st.K))


def test_zero_router_gives_exact_half_and_keeps():
    desc = CONFIGS["mini_fp32"]
    w = make_weights(desc, 41)
    prompt = make_prompt(desc.vocab, 37, 41)
    st = O.prefill_route(desc, w, torch.zeros(desc.n_layers, desc.d_model), prompt)
    assert torch.equal(st.rho, torch.full((desc.n_layers,), 0.5))
    assert st.mask.tolist() == [1] * desc.n_layers
    # the largest fp32 below 0.5 must skip (the decision is on the fp32 value)
    below = torch.nextafter(torch.tensor(0.5, dtype=torch.float32), torch.tensor(0.0))
    assert O.keep_decision(below) == 0 and O.keep_decision(torch.tensor(0.5)) == 1


def test_aligned_router_saturates():
    """A router pointing along (against) every token's stream vector gives rho -> 1 (0);
    rho always lies strictly inside (0, 1) and the mask is its threshold."""
    desc = CONFIGS["mini_fp32"]
    w = make_weights(desc, 43)
    prompt = make_prompt(desc.vocab, 24, 43)
    st0 = O.prefill_route(desc, w, torch.zeros(desc.n_layers, desc.d_model), prompt,
                          keep_router_inputs=True)
    mean_dir = torch.stack([h.mean(dim=0) for h in st0.router_in]).to(torch.float32)
    # layers >= 1 have a strong common component; layer 0 input is the raw embedding
    sign = torch.tensor([1.0, -1.0, 1.0])[:, None]
    router = sign * 8.0 * mean_dir / (mean_dir.norm(dim=1, keepdim=True) ** 2)
    st = O.prefill_route(desc, w, router, prompt)
    assert ((st.rho > 0) & (st.rho < 1)).all()
    assert st.mask.tolist() == [int(r >= 0.5) for r in st.rho.tolist()]
    assert st.rho[1] < 0.1 and st.mask[1] == 0 and st.rho[2] > 0.9 and st.mask[2] == 1
    assert O.compact_kept(st.mask) == [i for i in range(desc.n_layers) if st.mask[i]]


def test_router_score_matches_definition_by_hand():
    H = torch.tensor([[1.0, 2.0], [0.0, -1.0], [3.0, 0.5]], dtype=F64)
    wv = torch.tensor([0.5, -0.25], dtype=F64)
    zs = [0.0, 0.25, 1.375]
    ref = sum(1 / (1 + math.exp(-z)) for z in zs) / 3
    assert abs(float(O.router_score(H, wv)) - ref) < 1e-15


def test_prefill_ignores_routers_and_mask():
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 51)
    prompt = make_prompt(desc.vocab, 19, 51)
    a = O.prefill_route(desc, w, make_router(desc, 1), prompt)
    b = O.prefill_route(desc, w, make_router(desc, 2, std=5.0), prompt)
    assert torch.equal(a.logits, b.logits) and a.token == b.token
    assert all(torch.equal(x, y) for x, y in zip(a.K, b.K))
    assert all(torch.equal(x, y) for x, y in zip(a.V, b.V))
    assert not torch.equal(a.rho, b.rho)


def test_skipped_layer_leaves_hidden_and_kv_untouched_and_pruned_model_matches():
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 61)
    prompt = make_prompt(desc.vocab, 21, 61)
    st = O.prefill_route(desc, w, make_router(desc, 61), prompt)
    mask = [1, 0, 0, 1]
    st.set_mask(mask)
    kv_skipped = [(st.K[i].clone(), st.V[i].clone()) for i in (1, 2)]
    # pruned model: only the kept layers exist, and they get the same prefill KV
    kept = O.compact_kept(mask)
    pd = desc.with_(n_layers=len(kept))
    pw = dict(w)
    pw["layers"] = [w["layers"][i] for i in kept]
    pst = O.OracleState(K=[st.K[i].clone() for i in kept], V=[st.V[i].clone() for i in kept],
                        rho=st.rho[kept], mask=torch.ones(len(kept), dtype=torch.uint8),
                        n_prompt=st.n_prompt, pos=st.pos, hidden=st.hidden, logits=st.logits,
                        token=st.token)
    lg_m, tk_m = O.generate(desc, w, st, 4)
    lg_p, tk_p = O.generate(pd, pw, pst, 4)
    assert torch.equal(lg_m, lg_p) and tk_m == tk_p
    for (k0, v0), i in zip(kv_skipped, (1, 2)):
        assert torch.equal(k0, st.K[i]) and torch.equal(v0, st.V[i])
    assert st.K[0].shape[0] == prompt.numel() + 4
    # a layer skipped by earlier tokens cannot be switched back on: its KV has a hole
    st.set_mask([1, 1, 0, 1])
    with pytest.raises(ValueError):
        O.decode_step(desc, w, st, 5)


def test_rope_relative_position_and_norm():
    torch.manual_seed(0)
    q = torch.randn(1, 2, 16, dtype=F64)
    k = torch.randn(1, 2, 16, dtype=F64)
    def dot(m, n):
        return (O.rope(q, torch.tensor([m]), 10000.0) * O.rope(k, torch.tensor([n]), 10000.0)).sum(-1)
    assert torch.allclose(dot(7, 3), dot(104, 100), atol=1e-12)
    assert torch.allclose(dot(5, 5), (q * k).sum(-1), atol=1e-12)
    assert not torch.allclose(dot(7, 3), dot(3, 7), atol=1e-6)
    r = O.rope(q, torch.tensor([12345]), 10000.0)
    assert torch.allclose(r.norm(dim=-1), q.norm(dim=-1), atol=1e-12)
    assert torch.equal(O.rope(q, torch.tensor([0]), 10000.0), q)
    # first pair turns by exactly pos radians: position pi/2 is not an integer, so check 1 rad
    e = torch.zeros(1, 1, 4, dtype=F64); e[0, 0, 0] = 1.0
    r1 = O.rope(e, torch.tensor([1]), 10000.0)[0, 0]
    assert abs(float(r1[0]) - math.cos(1.0)) < 1e-15 and abs(float(r1[2]) - math.sin(1.0)) < 1e-15
    assert abs(float(r1[1])) < 1e-15 and abs(float(r1[3])) < 1e-15


def test_attention_special_cases():
    torch.manual_seed(1)
    n, Hq, Hkv, hd = 9, 4, 2, 8
    q = torch.randn(n, Hq, hd, dtype=F64)
    K = torch.randn(n, Hkv, hd, dtype=F64)
    V = torch.randn(n, Hkv, hd, dtype=F64)
    pos = torch.arange(n)
    a = O.attention_rows(q, K, V, pos, Hq // Hkv)
    # first row sees only key 0 -> returns V[0] of its KV head
    for h in range(Hq):
        assert torch.allclose(a[0, h], V[0, h // 2], atol=1e-14)
    # constant V -> output is that constant whatever the scores
    Vc = torch.ones_like(V) * 3.25
    assert torch.allclose(O.attention_rows(q, K, Vc, pos, 2), torch.full_like(q, 3.25), atol=1e-13)
    # causality: changing later keys does not change earlier rows
    K2 = K.clone(); K2[5:] += 10.0
    assert torch.equal(O.attention_rows(q, K2, V, pos, 2)[:5], a[:5])
    # library attention as a third opinion (MHA after repeating KV heads)
    ref = F.scaled_dot_product_attention(q.transpose(0, 1)[None], K.repeat_interleave(2, 1).transpose(0, 1)[None],
                                         V.repeat_interleave(2, 1).transpose(0, 1)[None], is_causal=True)[0]
    assert torch.allclose(a, ref.transpose(0, 1), atol=1e-12)


def test_norm_and_mlp_against_library():
    torch.manual_seed(2)
    x = torch.randn(5, 32, dtype=F64)
    g = torch.rand(32, dtype=F64) + 0.5
    assert torch.allclose(O.rmsnorm(x, g, 1e-5), F.rms_norm(x, (32,), g, 1e-5), atol=1e-14)
    wg, wu, wd = (torch.randn(48, 32, dtype=F64), torch.randn(48, 32, dtype=F64), torch.randn(32, 48, dtype=F64))
    ref = F.linear(F.silu(F.linear(x, wg)) * F.linear(x, wu), wd)
    assert torch.allclose(O.mlp(x, wg, wu, wd), ref, atol=1e-11)


def test_greedy_ties_go_to_lowest_index():
    lg = torch.tensor([0.1, 2.0, -1.0, 2.0, 2.0], dtype=torch.float32)
    assert O.greedy_token(lg) == 1


def test_kv_storage_rounding_is_bf16_for_bf16_models():
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 71)
    st = O.prefill_route(desc, w, make_router(desc, 71), make_prompt(desc.vocab, 5, 71))
    assert st.K[0].dtype == torch.bfloat16 and st.V[0].dtype == torch.bfloat16
    assert st.K[0].shape == (5, desc.n_kv_heads, desc.head_dim)


def test_router_parameter_fraction_matches_printed_values():
    path = os.path.join(os.path.dirname(__file__), "golden", "router_param_fraction.txt")
    printed = sorted(float(l.split()[1]) for l in open(path) if l.strip() and not l.startswith("#"))
    # public geometries of the two models the paper used
    llama3_8b = ModelDesc(32, 4096, 32, 8, 128, 14336, 128256)
    llama32_3b = ModelDesc(28, 3072, 24, 8, 128, 8192, 128256)
    def total(d, tied):
        return (d.n_layers * (d.layer_params + 2 * d.d_model) + d.d_model
                + d.vocab * d.d_model * (1 if tied else 2))
    fr = sorted([100.0 * make_router(llama3_8b, 0).numel() / total(llama3_8b, False),
                 100.0 * make_router(llama32_3b, 0).numel() / total(llama32_3b, True)])
    assert [round(x, 4) for x in fr] == printed


def test_skip_mask_generator_keeps_first_and_last():
    for seed in range(5):
        m = make_skip_mask(32, 16, seed)
        assert m[0] == 1 and m[-1] == 1 and int(m.sum()) == 16
    with pytest.raises(ValueError):
        make_skip_mask(4, 3, 0)


def test_kv_elision_drops_exactly_the_skipped_layers_and_changes_no_result():
    """Section 4.1 + 4.3: the decision of router i precedes layer i and is final, so the KV of a
    skipped layer is never read again.  Pins: same rho / mask / first token with and without
    elision; the kept layers' KV identical; decode identical; and the elided state is all a
    model pruned to the kept layers needs."""
    desc = CONFIGS["mini_bf16"]
    w = make_weights(desc, 71)
    prompt = make_prompt(desc.vocab, 23, 71)
    for seed in range(71, 120):                       # a router draw that keeps some layers and skips some
        router = make_router(desc, seed, std=5.0)
        full = O.prefill_route(desc, w, router, prompt)
        if 0 < int(full.mask.sum()) < desc.n_layers:
            break
    el = O.prefill_route(desc, w, router, prompt, elide_kv=True)
    assert torch.equal(full.rho, el.rho) and torch.equal(full.mask, el.mask)
    assert torch.equal(full.logits, el.logits) and full.token == el.token
    for i in range(desc.n_layers):
        if int(full.mask[i]):
            assert torch.equal(full.K[i], el.K[i]) and torch.equal(full.V[i], el.V[i])
        else:
            assert el.K[i] is None and el.V[i] is None
    kept = O.compact_kept(el.mask)
    pd = desc.with_(n_layers=len(kept))
    pw = dict(w)
    pw["layers"] = [w["layers"][i] for i in kept]
    pst = O.OracleState(K=[el.K[i].clone() for i in kept], V=[el.V[i].clone() for i in kept], rho=el.rho[kept],
                        mask=torch.ones(len(kept), dtype=torch.uint8), n_prompt=el.n_prompt, pos=el.pos,
                        hidden=el.hidden, logits=el.logits, token=el.token)
    lg_f, tk_f = O.generate(desc, w, full, 5)
    lg_e, tk_e = O.generate(desc, w, el, 5)
    lg_p, tk_p = O.generate(pd, pw, pst, 5)
    assert torch.equal(lg_f, lg_e) and tk_f == tk_e
    assert torch.equal(lg_e, lg_p) and tk_e == tk_p
    # a layer whose prompt KV was dropped cannot be switched on afterwards
    skipped = [i for i in range(desc.n_layers) if not int(el.mask[i])]
    m = el.mask.clone()
    m[skipped[0]] = 1
    el.set_mask(m)
    with pytest.raises(ValueError):
        O.decode_step(desc, w, el, 3)


def test_kv_elision_accounting():
    """Bytes by hand for the 8B shape: K and V of one token in one layer are 2 * 8 heads * 128 * 2 B =
    4 KiB, so a 1024-token prompt holds 128 MiB over 32 layers and 96 MiB when 8 layers are skipped
    (saving = skip fraction).  Slices are per layer: a batch stores the union of its kept layers."""
    desc = ModelDesc(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=14336,
                     vocab=128256, dtype="bf16")
    assert O.kv_bytes(desc, 1, 1) == 4096
    assert O.kv_bytes(desc, 32, 1024) == 128 << 20
    mask = make_skip_mask(32, 8, 5)
    stored = O.kv_layers_stored([mask])
    assert stored == [i for i in range(32) if mask[i]] and len(stored) == 24
    assert O.kv_bytes(desc, len(stored), 1024) == 96 << 20
    assert O.kv_bytes(desc, len(stored), 1024) / O.kv_bytes(desc, 32, 1024) == 1 - 8 / 32
    masks = [[1, 0, 0, 1, 0], [1, 1, 0, 0, 0], [0, 0, 0, 1, 0]]
    assert O.kv_layers_stored(masks) == [0, 1, 3]
    assert O.kv_layers_stored([[0, 0]]) == []

