"""Full-length decode attention (16 k context) on directly written KV: the cache of every layer is
filled with seeded synthetic keys / values through the test taps (no 16 k-token oracle prefill),
the sequence is declared that long, and decode steps are compared with the oracle holding the
same cache.  Covers many key tiles per wave, the maximum number of splits and page tables of a
thousand pages on all three decode paths."""
import pytest
import torch

from oracle import first_oracle as O
from synth import CONFIGS, make_prompt
from tests.gpu_util import build, logits_close
from tests.test_gpu_path import _decode, _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)


def _fill(ctx, st, desc, seq, n_ctx, seed):
    """Same synthetic cache on both sides: N(0, 0.5^2) rounded to the cache type."""
    g = torch.Generator().manual_seed(seed)
    ctx.set_seq_len(seq, n_ctx)
    for i in range(desc.n_layers):
        k = (torch.randn(n_ctx, desc.n_kv_heads, desc.head_dim, generator=g) * 0.5).to(torch.bfloat16)
        v = (torch.randn(n_ctx, desc.n_kv_heads, desc.head_dim, generator=g) * 0.5).to(torch.bfloat16)
        ctx.kv_write(seq, i, 0, k.float().cuda(), v.float().cuda())
        st.K[i], st.V[i] = k, v
    st.pos = n_ctx


@pytest.mark.parametrize("model,path,n_ctx", [("mini_hd128", 0, 16384), ("step_hd128", 1, 16384), ("step_hd64", 1, 5000)])
def test_decode_at_long_context_on_written_kv(model, path, n_ctx):
    desc = CONFIGS[model]
    prompt = make_prompt(desc.vocab, 24, 81)
    desc, w, router, ctx = build(model, 81, max_seq_len=n_ctx + 16)
    ctx.set_option(3, path)                               # per-op kernels / persistent kernel, or an error
    st = O.prefill_route(desc, w, router, prompt)
    _prefill(ctx, desc, [prompt])
    mask = [1] * desc.n_layers
    ctx.set_mask(0, mask)
    st.set_mask(mask)
    _fill(ctx, st, desc, 0, n_ctx, 82)
    n_steps = 3
    ref_lg, ref_tk = O.generate(desc, w, st, n_steps, forced=[5, 17, 1234 % desc.vocab])
    lg, tk = _decode(ctx, desc, [[5], [17], [1234 % desc.vocab]])
    for s in range(n_steps):
        ok, ma, rel = logits_close(lg[s, 0], ref_lg[s], desc.dtype)
        assert ok, (s, ma, rel)
    assert ctx.seq_len(0) == n_ctx + n_steps
    k, v = ctx.kv_read(0, desc.n_layers - 1, n_ctx, n_steps)
    kr = st.K[desc.n_layers - 1][n_ctx:].double()
    assert float((k.cpu().double() - kr).norm() / kr.norm()) <= 1.5e-2
    ctx.close()


def test_batched_decode_with_one_long_and_one_short_sequence():
    desc = CONFIGS["mini_hd128"]
    prompts = [make_prompt(desc.vocab, 24, 83), make_prompt(desc.vocab, 40, 84)]
    n_ctx = 9000
    desc, w, router, ctx = build("mini_hd128", 83, max_batch=2, max_seq_len=n_ctx + 16)
    ctx.set_option(6, 1)                                  # shared pass or an error
    sts = [O.prefill_route(desc, w, router, p) for p in prompts]
    _prefill(ctx, desc, prompts)
    masks = [[1, 0, 1], [1, 1, 1]]
    for b, m in enumerate(masks):
        ctx.set_mask(b, m)
        sts[b].set_mask(m)
    _fill(ctx, sts[0], desc, 0, n_ctx, 85)
    forced = [[7, 9], [11, 13], [15, 17]]
    refs = [O.generate(desc, w, sts[b], 3, forced=[row[b] for row in forced]) for b in range(2)]
    lg, tk = _decode(ctx, desc, forced, B=2)
    for b in range(2):
        for s in range(3):
            ok, ma, rel = logits_close(lg[s, b], refs[b][0][s], desc.dtype)
            assert ok, (b, s, ma, rel)
    assert [ctx.seq_len(0), ctx.seq_len(1)] == [n_ctx + 3, 43]
    ctx.close()


def test_batched_decode_with_the_8b_head_geometry_at_16k_keys():
    """The batched path's matrix-core attention (4 query heads per KV head, head dimension 128) with the 8B head counts
    (32 / 8) over 16 384 written positions, two sequences of very different length in one launch."""
    desc = CONFIGS["mini_8b_heads"]
    prompts = [make_prompt(desc.vocab, 24, 86), make_prompt(desc.vocab, 300, 87)]
    n_ctx = 16384
    desc, w, router, ctx = build("mini_8b_heads", 86, max_batch=2, max_seq_len=n_ctx + 16)
    ctx.set_option(6, 1)                                  # shared pass or an error
    sts = [O.prefill_route(desc, w, router, p) for p in prompts]
    _prefill(ctx, desc, prompts)
    masks = [[1, 1], [1, 1]]
    for b, m in enumerate(masks):
        ctx.set_mask(b, m)
        sts[b].set_mask(m)
    _fill(ctx, sts[0], desc, 0, n_ctx, 88)
    forced = [[7, 9], [11, 13], [15, 17]]
    refs = [O.generate(desc, w, sts[b], 3, forced=[row[b] for row in forced]) for b in range(2)]
    lg, tk = _decode(ctx, desc, forced, B=2)
    for b in range(2):
        for s in range(3):
            ok, ma, rel = logits_close(lg[s, b], refs[b][0][s], desc.dtype)
            assert ok, (b, s, ma, rel)
    assert [ctx.seq_len(0), ctx.seq_len(1)] == [n_ctx + 3, 303]
    k, v = ctx.kv_read(0, 1, n_ctx, 3)
    kr = sts[0].K[1][n_ctx:].double()
    assert float((k.cpu().double() - kr).norm() / kr.norm()) <= 1.5e-2
    ctx.close()
