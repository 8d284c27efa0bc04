"""Parity of the HIP prefill/route/decode path with the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import first_oracle as O
from synth import CONFIGS, make_prompt, make_router, make_skip_mask
from tests.gpu_util import TOL, build, logits_close, routers_with_margin, top2_gap

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)

MODELS = ["mini_fp32", "mini_bf16", "mini_hd128", "tiny"]
PROMPT = {"mini_fp32": 53, "mini_bf16": 70, "mini_hd128": 45, "tiny": 32}


def _dev_i32(x):
    return torch.as_tensor(x, dtype=torch.int32).cuda()


def _prefill(ctx, desc, prompts):
    B = len(prompts)
    ids = torch.cat(prompts).to(torch.int32).cuda()
    out = dict(rho=torch.zeros(B, desc.n_layers, device="cuda"),
               mask=torch.zeros(B, desc.n_layers, dtype=torch.uint8, device="cuda"),
               hidden=torch.zeros(B, desc.d_model, device="cuda"),
               logits=torch.zeros(B, desc.vocab, device="cuda"),
               token=torch.zeros(B, dtype=torch.int32, device="cuda"))
    ctx.prefill_route(ids, [p.numel() for p in prompts], **out)
    return {k: v.cpu() for k, v in out.items()}


def _decode(ctx, desc, tokens, B=1):
    """Teacher-forced decode: tokens[s][b] is the input of step s.  Returns logits [S,B,V], argmax [S,B]."""
    lg = torch.zeros(B, desc.vocab, device="cuda")
    tk = torch.zeros(B, dtype=torch.int32, device="cuda")
    tin = torch.zeros(B, dtype=torch.int32, device="cuda")
    L, T = [], []
    for row in tokens:
        tin.copy_(_dev_i32(row))
        ctx.decode_step(tin, lg, tk)
        ctx.sync()
        L.append(lg.cpu().clone())
        T.append(tk.cpu().clone())
    return torch.stack(L), torch.stack(T)


@pytest.mark.parametrize("model", MODELS)
def test_prefill_route_matches_oracle(model):
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, PROMPT[model], 7)
    from synth import make_weights
    w = make_weights(desc, 7)
    router = routers_with_margin(desc, w, [prompt], 7)
    desc, w, router, ctx = build(model, 7, max_seq_len=128, router=router)
    st = O.prefill_route(desc, w, router, prompt)
    got = _prefill(ctx, desc, [prompt])
    # router probabilities and the cached decisions
    assert float((got["rho"][0] - st.rho).abs().max()) <= (5e-4 if desc.dtype == "bf16" else 2e-6)   # (measured: up to 3.1e-4 at the 8B shape; the routers keep a margin of 2e-3)
    assert got["mask"][0].tolist() == st.mask.tolist()
    assert ctx.get_kept(0) == O.compact_kept(st.mask)
    assert ctx.seq_len(0) == prompt.numel()
    # last-position hidden state and first-token logits (full model: no skipping in prefill)
    ok, ma, rel = logits_close(got["logits"][0], st.logits, desc.dtype)
    assert ok, (ma, rel)
    h_rel = float((got["hidden"][0].double() - st.hidden).norm() / st.hidden.norm())
    assert h_rel <= TOL[desc.dtype]["rel"]
    if top2_gap(st.logits) > 2 * ma:              # decided beyond twice the measured logit error
        assert int(got["token"][0]) == st.token
    assert int(got["token"][0]) == int(torch.argmax(got["logits"][0]))
    # KV of every layer, every prompt position
    for i in range(desc.n_layers):
        k, v = ctx.kv_read(0, i, 0, prompt.numel())
        for a, b in ((k, st.K[i]), (v, st.V[i])):
            d = (a.cpu().double() - b.double())
            assert float(d.norm() / b.double().norm()) <= (1.5e-2 if desc.dtype == "bf16" else 1e-5)
    ctx.close()


@pytest.mark.parametrize("model", MODELS)
@pytest.mark.parametrize("mask_kind", ["routed", "interior", "all_keep", "all_skip"])
def test_decode_matches_oracle_teacher_forced(model, mask_kind):
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, PROMPT[model], 9)
    from synth import make_weights
    w = make_weights(desc, 9)
    router = routers_with_margin(desc, w, [prompt], 9)
    desc, w, router, ctx = build(model, 9, max_seq_len=128, router=router)
    st = O.prefill_route(desc, w, router, prompt)
    got = _prefill(ctx, desc, [prompt])
    L = desc.n_layers
    if mask_kind != "routed":
        mask = {"interior": [1] + [0] * (L - 2) + [1], "all_keep": [1] * L, "all_skip": [0] * L}[mask_kind]
        st.set_mask(mask)
        ctx.set_mask(0, mask)
    assert ctx.get_kept(0) == O.compact_kept(st.mask)
    n_steps = 20                                     # crosses a 16-token page boundary
    ref_lg, ref_tk = O.generate(desc, w, st, n_steps)
    inputs = [st.token] + ref_tk[:-1]
    lg, tk = _decode(ctx, desc, [[t] for t in inputs])
    checked = 0
    for s in range(n_steps):
        ok, ma, rel = logits_close(lg[s, 0], ref_lg[s], desc.dtype)
        assert ok, (s, ma, rel)
        assert int(tk[s, 0]) == int(torch.argmax(lg[s, 0]))
        if top2_gap(ref_lg[s]) > 2 * ma:           # decided beyond twice the measured logit error
            assert int(tk[s, 0]) == ref_tk[s]
            checked += 1
    assert checked >= (3 * n_steps) // 4
    assert ctx.seq_len(0) == prompt.numel() + n_steps
    # kept layers hold KV for the new positions, equal to the oracle's
    for i in O.compact_kept(st.mask):
        k, v = ctx.kv_read(0, i, prompt.numel(), n_steps)
        kr = st.K[i][prompt.numel():].double()
        assert float((k.cpu().double() - kr).norm() / kr.norm()) <= (1.5e-2 if desc.dtype == "bf16" else 1e-5)
    ctx.close()


@pytest.mark.parametrize("model", ["mini_bf16", "mini_hd128", "mini_fp32"])
def test_decode_alone_is_tight_when_given_the_oracle_kv(model):
    """With the oracle's prompt KV loaded into the pages the decode kernels see exactly the
    oracle's inputs, so only fp32 summation order separates the two."""
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, PROMPT[model], 11)
    desc, w, router, ctx = build(model, 11, max_seq_len=128)
    st = O.prefill_route(desc, w, router, prompt)
    _prefill(ctx, desc, [prompt])
    for i in range(desc.n_layers):
        ctx.kv_write(0, i, 0, st.K[i].float().cuda().contiguous(), st.V[i].float().cuda().contiguous())
        k, v = ctx.kv_read(0, i, 0, prompt.numel())
        assert torch.equal(k.cpu(), st.K[i].float()) and torch.equal(v.cpu(), st.V[i].float())
    mask = make_skip_mask(desc.n_layers, 1, 11).tolist()
    st.set_mask(mask)
    ctx.set_mask(0, mask)
    ref_lg, ref_tk = O.generate(desc, w, st, 6)
    lg, tk = _decode(ctx, desc, [[t] for t in [st.token] + ref_tk[:-1]])
    err = float((lg[:, 0].double() - ref_lg.double()).abs().max())
    # bf16 KV: a new key/value can round to the neighbouring bf16 on one side only
    assert err <= (3e-3 if desc.dtype == "bf16" else 2e-5), err
    ctx.close()


def test_all_skip_is_embedding_norm_head_and_hidden_is_bit_identical():
    desc, w, router, ctx = build("mini_bf16", 13, max_seq_len=128)
    prompt = make_prompt(desc.vocab, 40, 13)
    _prefill(ctx, desc, [prompt])
    ctx.set_mask(0, [0] * desc.n_layers)
    assert ctx.get_kept(0) == []
    sent = torch.full((8, desc.n_kv_heads, desc.head_dim), -3.0, device="cuda")
    for i in range(desc.n_layers):                               # define the unused tail of the last page
        ctx.kv_write(0, i, 40, sent, sent)
    before = [tuple(t.clone() for t in ctx.kv_read(0, i, 0, 48)) for i in range(desc.n_layers)]
    tok = 123
    lg, tk = _decode(ctx, desc, [[tok]])
    h = ctx.get_hidden().cpu()
    assert torch.equal(h[0], w["embed"][tok].float())            # residual passed through untouched
    e = w["embed"][tok].double()
    x = e / torch.sqrt((e * e).mean() + desc.rms_eps) * w["final_norm"].double()
    ref = w["lm_head"].double() @ x
    assert float((lg[0, 0].double() - ref).abs().max()) <= 1e-5
    for i in range(desc.n_layers):                               # no KV byte of any layer changed
        k, v = ctx.kv_read(0, i, 0, 48)
        assert torch.equal(k, before[i][0]) and torch.equal(v, before[i][1])
    ctx.close()


def test_skipped_layers_never_touch_their_kv_and_kept_layers_append():
    desc, w, router, ctx = build("mini_bf16", 15, max_seq_len=128)
    prompt = make_prompt(desc.vocab, 30, 15)
    _prefill(ctx, desc, [prompt])
    mask = [1, 0, 0, 1]
    ctx.set_mask(0, mask)
    n0 = prompt.numel()
    # sentinel in the slots decode would write (positions 30, 31 lie in an allocated page)
    sent = torch.full((2, desc.n_kv_heads, desc.head_dim), -7.0, device="cuda")
    for i in range(desc.n_layers):
        ctx.kv_write(0, i, n0, sent, sent)
    before = [tuple(t.clone() for t in ctx.kv_read(0, i, 0, 32)) for i in range(desc.n_layers)]
    _decode(ctx, desc, [[5], [6]])
    for i in range(desc.n_layers):
        k, v = ctx.kv_read(0, i, 0, 32)
        if mask[i]:
            assert torch.equal(k[:n0], before[i][0][:n0]) and not torch.equal(k[n0:], before[i][0][n0:])
            assert float(v[n0:].max()) != -7.0 or float(v[n0:].min()) != -7.0
        else:
            assert torch.equal(k, before[i][0]) and torch.equal(v, before[i][1])
    ctx.close()


def test_zero_router_gives_exactly_half_and_keeps_every_layer():
    desc = CONFIGS["mini_bf16"]
    desc, w, router, ctx = build("mini_bf16", 17, max_seq_len=128,
                                 router=torch.zeros(desc.n_layers, desc.d_model))
    got = _prefill(ctx, desc, [make_prompt(desc.vocab, 37, 17)])
    assert torch.equal(got["rho"][0], torch.full((desc.n_layers,), 0.5))
    assert got["mask"][0].tolist() == [1] * desc.n_layers
    ctx.close()


def test_prefill_is_independent_of_the_routers():
    outs = []
    for rs in (1, 2):
        desc = CONFIGS["mini_bf16"]
        desc, w, router, ctx = build("mini_bf16", 19, max_seq_len=128, router=make_router(desc, rs, std=3.0))
        got = _prefill(ctx, desc, [make_prompt(desc.vocab, 33, 19)])
        kv = [ctx.kv_read(0, i, 0, 33) for i in range(desc.n_layers)]
        outs.append((got, kv))
        ctx.close()
    assert torch.equal(outs[0][0]["logits"], outs[1][0]["logits"])
    assert all(torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) for a, b in zip(outs[0][1], outs[1][1]))
    assert not torch.equal(outs[0][0]["rho"], outs[1][0]["rho"])


def test_page_permutation_and_graph_replay_do_not_change_a_bit():
    prompt = make_prompt(CONFIGS["mini_bf16"].vocab, 50, 21)
    runs = []
    for variant in ("plain", "shuffled_pages", "eager"):
        desc, w, router, ctx = build("mini_bf16", 21, max_seq_len=128)
        if variant == "shuffled_pages":
            rng = np.random.default_rng(0)
            ctx.set_page_order(rng.permutation(ctx.num_pages()).tolist())
        if variant == "eager":
            ctx.set_option(1, 0)
        got = _prefill(ctx, desc, [prompt])
        ctx.set_mask(0, [1, 0, 1, 1])
        lg, tk = _decode(ctx, desc, [[int(got["token"][0])]] + [[t] for t in range(3, 22)])
        runs.append((got["logits"], lg, tk))
        ctx.close()
    for r in runs[1:]:
        assert torch.equal(runs[0][0], r[0]) and torch.equal(runs[0][1], r[1]) and torch.equal(runs[0][2], r[2])


@pytest.mark.parametrize("model,T", [("mini_bf16", 203), ("mini_hd128", 97), ("mini_hd128", 1)])
def test_prompt_attention_on_matrix_cores_agrees_with_the_plain_kernel(model, T):
    """Option 7: 1 = tiled MFMA kernel (default), 0 = plain fp32 kernel; same cache, same
    logits up to the 16-bit split of queries and probabilities."""
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, T, 77)
    outs = {}
    for kind in (1, 0):
        desc, w, router, ctx = build(model, 77, max_seq_len=T + 8)
        ctx.set_option(7, kind)
        outs[kind] = _prefill(ctx, desc, [prompt])
        outs[kind]["k_last"] = ctx.kv_read(0, desc.n_layers - 1, 0, T)[0].float().cpu()
        ctx.close()
    scale = float(outs[0]["logits"].abs().max())
    assert float((outs[1]["logits"] - outs[0]["logits"]).abs().max()) <= 2e-3 * max(scale, 1.0)
    assert float((outs[1]["rho"] - outs[0]["rho"]).abs().max()) <= 1e-4
    assert float((outs[1]["k_last"] - outs[0]["k_last"]).abs().max()) <= 2e-2 * float(outs[0]["k_last"].abs().max())
    st = O.prefill_route(desc, w, router, prompt)
    ok, ma, rel = logits_close(outs[1]["logits"][0], st.logits, desc.dtype)
    assert ok, (ma, rel)


def test_batch_of_sequences_equals_each_sequence_alone():
    desc = CONFIGS["mini_bf16"]
    prompts = [make_prompt(desc.vocab, n, 30 + i) for i, n in enumerate((17, 64, 33))]
    masks = [[1, 1, 1, 1], [1, 0, 1, 1], [1, 0, 0, 1]]
    steps = [[3 + s, 40 + s, 900 + s] for s in range(18)]
    desc, w, router, ctx = build("mini_bf16", 23, max_batch=3, max_seq_len=128)
    ctx.set_option(6, 0)        # one pass per sequence: the same kernels as a lone sequence, so every bit agrees
    got = _prefill(ctx, desc, prompts)
    for b, m in enumerate(masks):
        ctx.set_mask(b, m)
    lg, tk = _decode(ctx, desc, steps, B=3)
    assert [ctx.seq_len(b) for b in range(3)] == [p.numel() + 18 for p in prompts]
    ctx.close()
    for b in range(3):
        desc, w, router, c1 = build("mini_bf16", 23, max_batch=1, max_seq_len=128)
        g1 = _prefill(c1, desc, [prompts[b]])
        c1.set_mask(0, masks[b])
        lg1, tk1 = _decode(c1, desc, [[row[b]] for row in steps])
        assert torch.equal(g1["logits"][0], got["logits"][b]) and torch.equal(g1["rho"][0], got["rho"][b])
        assert torch.equal(lg1[:, 0], lg[:, b]) and torch.equal(tk1[:, 0], tk[:, b])
        c1.close()
    # and against the oracle for the ragged batch (sequence 1, masked)
    st = O.prefill_route(desc, w, router, prompts[1])
    st.set_mask(masks[1])
    ref_lg, _ = O.generate(desc, w, st, 18, forced=[row[1] for row in steps])
    ok, ma, rel = logits_close(lg[:, 1], ref_lg, desc.dtype)
    assert ok, (ma, rel)


def test_state_and_capacity_errors():
    import paper_2410_12513_amd as P
    desc, w, router, ctx = build("mini_bf16", 25, max_batch=1, max_seq_len=40)
    tin = _dev_i32([1]); tk = _dev_i32([0])
    with pytest.raises(P.FirstError) as e:
        ctx.decode_step(tin, None, tk)                      # decode before prefill
    assert e.value.code == -2
    with pytest.raises(P.FirstError) as e:
        ctx.set_mask(0, [1] * desc.n_layers)
    assert e.value.code == -2
    ids = make_prompt(desc.vocab, 64, 1).cuda()
    with pytest.raises(P.FirstError) as e:
        ctx.prefill_route(ids, [40])                        # no room for a generated token
    assert e.value.code == -3
    with pytest.raises(P.FirstError) as e:
        ctx.prefill_route(ids, [20, 20])                    # batch above max_batch
    assert e.value.code == -3
    ctx.prefill_route(ids, [38])
    ctx.set_mask(0, [1, 0, 1, 1])
    ctx.decode_step(tin, None, tk)
    with pytest.raises(P.FirstError) as e:
        ctx.set_mask(0, [1, 1, 1, 1])                       # re-enabling a layer after decode began
    assert e.value.code == -2
    ctx.set_mask(0, [1, 0, 0, 1])                           # clearing bits stays legal
    ctx.decode_step(tin, None, tk)
    with pytest.raises(P.FirstError) as e:
        ctx.decode_step(tin, None, tk)                      # sequence is full (40 tokens)
    assert e.value.code == -3
    ctx.sync()
    assert ctx.seq_len(0) == 40
    ctx.close()
