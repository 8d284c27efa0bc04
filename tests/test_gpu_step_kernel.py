"""The persistent whole-step decode kernel (one launch per token) against the oracle and
against the per-op kernels, through the C ABI.  Option 3 = 1 makes the library refuse to
fall back, so these tests cannot pass on another path."""
import pytest
import torch

from oracle import first_oracle as O
from synth import CONFIGS, make_prompt, make_skip_mask, make_weights
from tests.gpu_util import TOL, build, logits_close, routers_with_margin, top2_gap
from tests.test_gpu_path import _decode, _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)

OPT_DECODE_PATH = 3


@pytest.mark.parametrize("model,n_prompt", [("step_hd128", 150), ("step_hd64", 70), ("step_g2", 200),
                                            ("step_mha", 65), ("step_hd128", 700), ("step_3k", 90)])
@pytest.mark.parametrize("mask_kind", ["interior", "all_keep", "all_skip"])
def test_step_kernel_matches_oracle(model, n_prompt, mask_kind):
    desc = CONFIGS[model]
    if n_prompt > 300 and mask_kind != "interior":
        pytest.skip("long prompt is run once")
    prompt = make_prompt(desc.vocab, n_prompt, 41)
    desc, w, router, ctx = build(model, 41, max_seq_len=n_prompt + 40)
    ctx.set_option(OPT_DECODE_PATH, 1)
    st = O.prefill_route(desc, w, router, prompt)
    _prefill(ctx, desc, [prompt])
    L = desc.n_layers
    mask = {"interior": [1] + [0] * (L - 2) + [1] if L > 2 else [0, 1], "all_keep": [1] * L, "all_skip": [0] * L}[mask_kind]
    st.set_mask(mask)
    ctx.set_mask(0, mask)
    n_steps = 20
    ref_lg, ref_tk = O.generate(desc, w, st, n_steps)
    lg, tk = _decode(ctx, desc, [[t] for t in [st.token] + ref_tk[:-1]])
    checked = 0
    for s in range(n_steps):
        ok, ma, rel = logits_close(lg[s, 0], ref_lg[s], desc.dtype)
        assert ok, (s, ma, rel)
        assert int(tk[s, 0]) == int(torch.argmax(lg[s, 0]))
        if top2_gap(ref_lg[s]) > 2 * ma:
            assert int(tk[s, 0]) == ref_tk[s]
            checked += 1
    assert checked >= (3 * n_steps) // 4
    assert ctx.seq_len(0) == n_prompt + n_steps
    for i in O.compact_kept(st.mask):
        k, v = ctx.kv_read(0, i, n_prompt, n_steps)
        kr = st.K[i][n_prompt:].double()
        assert float((k.cpu().double() - kr).norm() / kr.norm()) <= 1.5e-2
    ctx.close()


@pytest.mark.parametrize("model", ["step_hd128", "step_hd64"])
def test_step_kernel_agrees_with_per_op_kernels_and_is_reproducible(model):
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, 130, 43)
    mask = make_skip_mask(desc.n_layers, 1 if desc.n_layers > 2 else 0, 43).tolist()
    inputs = [[int(t)] for t in make_prompt(desc.vocab, 24, 44)]
    runs = {}
    for name, path, graph in (("ops", 0, 1), ("step", 1, 1), ("step_again", 1, 1), ("step_eager", 1, 0)):
        desc, w, router, ctx = build(model, 43, max_seq_len=200)
        ctx.set_option(OPT_DECODE_PATH, path)
        ctx.set_option(1, graph)
        _prefill(ctx, desc, [prompt])
        ctx.set_mask(0, mask)
        lg, tk = _decode(ctx, desc, inputs)
        h = ctx.get_hidden().cpu()
        runs[name] = (lg, tk, h)
        ctx.close()

    def same(a, b):
        return torch.equal(runs[a][0], runs[b][0]) and torch.equal(runs[a][1], runs[b][1]) and torch.equal(runs[a][2], runs[b][2])

    # fixed summation orders everywhere: run to run, and graph replay against eager launches
    assert same("step", "step_again") and same("step", "step_eager")
    # same arithmetic up to fp32 summation order
    assert float((runs["step"][0] - runs["ops"][0]).abs().max()) <= 3e-3   # a new K/V may round to the neighbouring bf16
    assert float((runs["step"][2] - runs["ops"][2]).abs().max()) <= 3e-3 * float(runs["ops"][2].abs().max())


def test_step_kernel_alternating_with_the_per_op_kernels_and_new_sequences():
    """The tagged exchange keeps state from launch to launch (the tags of the latest writes).  Steps of
    the per-op kernels in between, a new prefill and a different mask must not disturb it."""
    model = "step_hd128"
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, 90, 61)
    inputs = [[int(t)] for t in make_prompt(desc.vocab, 18, 62)]
    masks = [make_skip_mask(desc.n_layers, 1, 61).tolist(), [1] * desc.n_layers]

    def run(paths):
        desc_, w, router, ctx = build(model, 61, max_seq_len=160)
        out = []
        for mask in masks:                              # second round: new sequence in the same context
            _prefill(ctx, desc_, [prompt])
            ctx.set_mask(0, mask)
            for i, tok in enumerate(inputs):
                ctx.set_option(OPT_DECODE_PATH, paths[i % len(paths)])
                lg, tk = _decode(ctx, desc_, [tok])
                out.append(lg[0, 0].clone())
        ctx.close()
        return torch.stack(out)

    mixed, only_step, only_ops = run([1, 1, 0, 1, 0, 0, 1]), run([1]), run([0])
    assert float((only_step - only_ops).abs().max()) <= 3e-3
    assert float((mixed - only_ops).abs().max()) <= 3e-3
    assert float((mixed - only_step).abs().max()) <= 3e-3


def test_step_kernel_all_skip_leaves_hidden_bit_identical_and_kv_untouched():
    desc, w, router, ctx = build("step_hd128", 45, max_seq_len=128)
    ctx.set_option(OPT_DECODE_PATH, 1)
    prompt = make_prompt(desc.vocab, 40, 45)
    _prefill(ctx, desc, [prompt])
    ctx.set_mask(0, [1, 0, 0])
    sent = torch.full((8, desc.n_kv_heads, desc.head_dim), -3.0, device="cuda")
    for i in range(desc.n_layers):
        ctx.kv_write(0, i, 40, sent, sent)
    before = [tuple(t.clone() for t in ctx.kv_read(0, i, 0, 48)) for i in range(desc.n_layers)]
    _decode(ctx, desc, [[7], [9]])
    for i in (1, 2):
        k, v = ctx.kv_read(0, i, 0, 48)
        assert torch.equal(k, before[i][0]) and torch.equal(v, before[i][1])
    k, v = ctx.kv_read(0, 0, 0, 48)
    assert torch.equal(k[:40], before[0][0][:40]) and float(k[40:42].max()) != -3.0
    ctx.set_mask(0, [0, 0, 0])
    _decode(ctx, desc, [[123]])
    assert torch.equal(ctx.get_hidden().cpu()[0], w["embed"][123].float())
    ctx.close()


def test_step_kernel_is_refused_when_the_model_does_not_fit():
    import paper_2410_12513_amd as P
    desc, w, router, ctx = build("mini_bf16", 47, max_seq_len=64)
    ctx.set_option(OPT_DECODE_PATH, 1)
    _prefill(ctx, desc, [make_prompt(desc.vocab, 20, 47)])
    tin = torch.tensor([1], dtype=torch.int32, device="cuda")
    with pytest.raises(P.FirstError) as e:
        ctx.decode_step(tin, None, tin)
    assert e.value.code == -2
    ctx.set_option(OPT_DECODE_PATH, -1)
    ctx.decode_step(tin, None, tin)          # automatic choice falls back to the per-op kernels
    ctx.sync()
    ctx.close()


def test_step_kernel_long_run_is_reproducible_and_never_gives_up():
    """1500 free-running steps twice (each step feeds its own token): identical token streams,
    finite logits, and first_sync reports no barrier that gave up."""
    desc = CONFIGS["step_hd128"]
    prompt = make_prompt(desc.vocab, 33, 51)
    streams = []
    for run in range(2):
        desc, w, router, ctx = build("step_hd128", 51, max_seq_len=33 + 1500 + 8)
        ctx.set_option(OPT_DECODE_PATH, 1)
        got = _prefill(ctx, desc, [prompt])
        ctx.set_mask(0, [1, 0, 1])
        tok = got["token"].to(torch.int32).cuda()
        hist = torch.zeros(1500, dtype=torch.int32, device="cuda")
        lg = torch.zeros(1, desc.vocab, device="cuda")
        for s in range(1500):
            ctx.decode_step(tok, lg, tok)
            ctx.sync()                           # raises if a grid barrier gave up
            hist[s:s + 1].copy_(tok)
        assert bool(torch.isfinite(lg).all())
        assert ctx.seq_len(0) == 33 + 1500
        streams.append(hist.cpu())
        ctx.close()
    assert torch.equal(streams[0], streams[1])


@pytest.mark.parametrize("model,n_prompt", [("step_hd128", 150), ("step_hd64", 700)])
def test_step_kernel_gives_up_in_an_orderly_way_and_recovers(model, n_prompt):
    """A wait between workgroups that gives up: forced from the host with a poll limit of 0 (every first unsuccessful poll
    gives up), so nothing has to go wrong for it.  Every wave leaves, the launch ends, the next synchronising call
    reports the error once and resets the exchange state; after a new prefill the context decodes exactly what an
    untouched twin decodes."""
    import paper_2410_12513_amd as P
    prompt = make_prompt(CONFIGS[model].vocab, n_prompt, 57)
    outs = []
    for provoke in (False, True):
        desc, w, router, ctx = build(model, 57, max_seq_len=n_prompt + 40)
        ctx.set_option(OPT_DECODE_PATH, 1)
        got = _prefill(ctx, desc, [prompt])
        tok = got["token"].to(torch.int32).cuda()
        if provoke:
            for use_graph in (1, 0):
                ctx.set_option(1, use_graph)
                ctx.set_option(10, 0)                     # STEP_POLL_LIMIT: give up at the first unsuccessful poll
                ctx.decode_step(tok, None, tok.clone())
                with pytest.raises(P.FirstError) as e:
                    ctx.sync()
                assert e.value.code == -4 and "gave up" in str(e.value)
                ctx.sync()                                # reported once; the limit went with the error
                got = _prefill(ctx, desc, [prompt])
                tok = got["token"].to(torch.int32).cuda()
            ctx.set_option(1, 1)
        lg = torch.zeros(1, desc.vocab, device="cuda")
        hist = []
        for s in range(12):
            ctx.decode_step(tok, lg, tok)
            ctx.sync()
            hist.append((int(tok[0]), lg.clone()))
        outs.append(hist)
        assert ctx.seq_len(0) == n_prompt + 12
        ctx.close()
    for (ta, la), (tb, lb) in zip(*outs):
        assert ta == tb and torch.equal(la, lb)
