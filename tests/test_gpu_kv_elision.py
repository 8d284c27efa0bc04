"""Skip-aware KV elision (kv_layer_slots): only layers some live sequence keeps own a slice of
the KV pool.  Through the C ABI, against the oracle's `elide_kv` prefill and against a context
without elision (bit-identical), on the persistent kernel, the per-op kernels and the batched path."""
import pytest
import torch

import paper_2410_12513_amd as P
from oracle import first_oracle as O
from synth import CONFIGS, make_prompt, make_weights
from tests.gpu_util import build, logits_close, routers_with_margin, top2_gap
from tests.test_gpu_path import _decode, _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)

OPT_DECODE_PATH = 3
OPT_BATCH_PATH = 6


def _setup(model, n_layers, lens, want, seed):
    desc = CONFIGS[model].with_(n_layers=n_layers)
    w = make_weights(desc, seed)
    prompts = [make_prompt(desc.vocab, n, seed + 10 * b) for b, n in enumerate(lens)]
    router = routers_with_margin(desc, w, prompts, seed, want=want, max_tries=400)
    return desc, w, prompts, router


@pytest.mark.parametrize("model,path", [("step_hd128", 1), ("mini_bf16", 0)])
def test_elided_context_matches_oracle_and_the_full_context(model, path):
    want = [[1, 0, 1, 0, 0, 1]]
    desc, w, prompts, router = _setup(model, 6, [77], want, 81)
    n_steps = 12
    st = O.prefill_route(desc, w, router, prompts[0], elide_kv=True)
    assert st.mask.tolist() == want[0]
    ref_lg, ref_tk = O.generate(desc, w, st, n_steps)
    inputs = [[t] for t in [st.token] + ref_tk[:-1]]
    runs = {}
    for name, slots in (("full", 0), ("elided", 3)):
        _, _, _, ctx = build(model, 81, max_seq_len=128, router=router, desc=desc, kv_layer_slots=slots)
        ctx.set_option(OPT_DECODE_PATH, path)
        got = _prefill(ctx, desc, prompts)
        assert got["mask"][0].tolist() == want[0]
        lg, tk = _decode(ctx, desc, inputs)
        runs[name] = (got["logits"], got["rho"], lg, tk, ctx.kv_usage(), ctx.num_pages())
        if name == "elided":
            assert ctx.get_kept(0) == [0, 2, 5]
            for s in range(n_steps):
                ok, ma, rel = logits_close(lg[s, 0], ref_lg[s], desc.dtype)
                assert ok, (s, ma, rel)
                if top2_gap(ref_lg[s]) > 2 * ma:
                    assert int(tk[s, 0]) == ref_tk[s]
            for i in (0, 2, 5):                                   # stored layers: prompt and generated positions
                k, v = ctx.kv_read(0, i, 0, 77 + n_steps)
                for a, b in ((k, st.K[i]), (v, st.V[i])):
                    assert float((a.cpu().double() - b.double()).norm() / b.double().norm()) <= 1.5e-2
            for i in (1, 3, 4):                                   # elided layers: no KV to read, cannot be switched on
                with pytest.raises(P.FirstError) as e:
                    ctx.kv_read(0, i, 0, 4)
                assert e.value.code == -2
                m = list(want[0]); m[i] = 1
                with pytest.raises(P.FirstError) as e:
                    ctx.set_mask(0, m)
                assert e.value.code == -2
            ctx.set_mask(0, [1, 0, 0, 0, 0, 1])                   # clearing a bit stays legal
            st.set_mask([1, 0, 0, 0, 0, 1])
            lg2, tk2 = O.decode_step(desc, w, st, 5)
            lgg, _ = _decode(ctx, desc, [[5]])
            ok, ma, rel = logits_close(lgg[0, 0], lg2, desc.dtype)
            assert ok, (ma, rel)
        ctx.close()
    f, e = runs["full"], runs["elided"]
    assert torch.equal(f[0], e[0]) and torch.equal(f[1], e[1]) and torch.equal(f[2], e[2]) and torch.equal(f[3], e[3])
    # memory: 3 slots + 1 scratch slice against 6 slices; the oracle's count of stored layers
    assert e[4][1:] == (3, len(O.kv_layers_stored([want[0]]))) and f[4][1:] == (6, 6)
    assert e[4][0] * 6 == f[4][0] * 4
    assert f[4][0] == O.kv_bytes(desc, 6, 16 * f[5])                      # pages of 16 tokens


def test_more_kept_layers_than_slots_is_a_capacity_error():
    want = [[1, 1, 0, 1]]
    desc, w, prompts, router = _setup("mini_bf16", 4, [40], want, 83)
    _, _, _, ctx = build("mini_bf16", 83, max_seq_len=64, router=router, desc=desc, kv_layer_slots=2)
    with pytest.raises(P.FirstError) as e:
        _prefill(ctx, desc, prompts)
    assert e.value.code == -3
    tin = torch.tensor([1], dtype=torch.int32, device="cuda")
    with pytest.raises(P.FirstError) as e:                        # no sequence became live
        ctx.decode_step(tin, None, tin)
    assert e.value.code == -2
    ctx.close()
    _, _, _, ctx = build("mini_bf16", 83, max_seq_len=64, router=router, desc=desc, kv_layer_slots=3)
    assert _prefill(ctx, desc, prompts)["mask"][0].tolist() == want[0]
    assert ctx.kv_usage()[1:] == (3, 3)
    ctx.close()


@pytest.mark.parametrize("batch_path", [1, 0])
def test_batch_shares_slices_per_layer_and_a_new_prefill_starts_over(batch_path):
    """Three sequences with different masks: slices = union of the kept layers.  Then a second
    prefill in the same context with other prompts (other masks): the slices are handed out anew."""
    want = [[1, 0, 0, 1, 0], [1, 1, 0, 0, 0], [0, 0, 0, 1, 0]]
    desc, w, prompts, router = _setup("step_hd128", 5, [50, 33, 90], want, 85)
    n_steps = 6
    _, _, _, ctx = build("step_hd128", 85, max_batch=3, max_seq_len=128, router=router, desc=desc, kv_layer_slots=4)
    _, _, _, full = build("step_hd128", 85, max_batch=3, max_seq_len=128, router=router, desc=desc)
    for c in (ctx, full):
        c.set_option(OPT_BATCH_PATH, batch_path)
    for round_, order in enumerate(([0, 1, 2], [2, 0])):
        ps = [prompts[b] for b in order]
        states = [O.prefill_route(desc, w, router, p, elide_kv=True) for p in ps]
        assert [s.mask.tolist() for s in states] == [want[b] for b in order]
        refs = [O.generate(desc, w, s, n_steps) for s in states]
        B = len(ps)
        steps = [[(states[b].token if s == 0 else refs[b][1][s - 1]) for b in range(B)] for s in range(n_steps)]
        got = _prefill(ctx, desc, ps)
        got_full = _prefill(full, desc, ps)
        assert got["mask"].tolist() == [want[b] for b in order]
        stored = O.kv_layers_stored([want[b] for b in order])
        assert ctx.kv_usage()[2] == len(stored)
        lg, tk = _decode(ctx, desc, steps, B=B)
        lg_full, tk_full = _decode(full, desc, steps, B=B)
        assert torch.equal(got["logits"], got_full["logits"]) and torch.equal(lg, lg_full) and torch.equal(tk, tk_full)
        for b in range(B):
            for s in range(n_steps):
                ok, ma, rel = logits_close(lg[s, b], refs[b][0][s], desc.dtype)
                assert ok, (round_, b, s, ma, rel)
    ctx.close()
    full.close()
