"""Decode of a batch with heterogeneous skip masks through the shared-pass path (per layer, the
sequences that keep it go through its weights together), against the oracle run on each
sequence alone.  Option 6 = 1 makes the library refuse any other path.  Shapes are reduced
versions of the batch-16 / mixed-mask and the batch-4 / long-context workloads."""
import pytest
import torch

from oracle import first_oracle as O
from synth import CONFIGS, make_prompt, make_skip_mask
from tests.gpu_util import build, logits_close, top2_gap
from tests.test_gpu_path import _decode, _prefill

pytestmark = pytest.mark.gpu
torch.set_grad_enabled(False)

OPT_BATCH_PATH = 6


def _masks(L, B, seed):
    """Per-sequence masks with different skip counts (0 .. L-2 interior layers), first/last kept."""
    out = []
    for b in range(B):
        k = b % max(1, L - 1)
        out.append(make_skip_mask(L, min(k, max(0, L - 2)), seed + b).tolist())
    return out


def _run(model, lens, n_steps, seed, page=16, splits=0, masks=None):
    desc = CONFIGS[model]
    B = len(lens)
    prompts = [make_prompt(desc.vocab, n, seed + 10 * b) for b, n in enumerate(lens)]
    desc, w, router, ctx = build(model, seed, max_batch=B, max_seq_len=max(lens) + n_steps + 8, page=page)
    ctx.set_option(OPT_BATCH_PATH, 1)
    ctx.set_option(2, splits)
    _prefill(ctx, desc, prompts)
    masks = masks or _masks(desc.n_layers, B, seed)
    for b, m in enumerate(masks):
        ctx.set_mask(b, m)
    states, refs = [], []
    for b in range(B):
        st = O.prefill_route(desc, w, router, prompts[b])
        st.set_mask(masks[b])
        states.append(st)
        refs.append(O.generate(desc, w, st, n_steps))          # greedy, per sequence
    # teacher-forced with the oracle's own tokens so that every sequence follows its reference
    steps = [[(states[b].token if s == 0 else refs[b][1][s - 1]) for b in range(B)] for s in range(n_steps)]
    lg, tk = _decode(ctx, desc, steps, B=B)
    worst, checked = 0.0, 0
    for b in range(B):
        for s in range(n_steps):
            ok, ma, rel = logits_close(lg[s, b], refs[b][0][s], desc.dtype)
            assert ok, (b, s, ma, rel)
            worst = max(worst, ma)
            assert int(tk[s, b]) == int(torch.argmax(lg[s, b]))
            if top2_gap(refs[b][0][s]) > 2 * ma:
                assert int(tk[s, b]) == refs[b][1][s]
                checked += 1
        assert ctx.seq_len(b) == lens[b] + n_steps
        for i in O.compact_kept(states[b].mask):
            k, v = ctx.kv_read(b, i, lens[b], n_steps)
            kr = states[b].K[i][lens[b]:].double()
            assert float((k.cpu().double() - kr).norm() / kr.norm()) <= 1.5e-2
    assert checked >= (3 * B * n_steps) // 4
    ctx.close()
    return worst


def test_batch16_mixed_masks_matches_oracle_per_sequence():
    lens = [21 + 7 * b for b in range(16)]                      # ragged prompts, several KV pages each
    _run("mini_bf16", lens, 6, 61)                               # d_ffn = 1416: ragged last MFMA step


def test_batch16_wide_model_matches_oracle():
    _run("step_hd128", [40 + 3 * b for b in range(16)], 4, 63)  # widths 2048 / 4096, K split over waves


def test_batch4_long_context_matches_oracle():
    _run("mini_hd128", [2048, 1900, 2048, 1777], 4, 65)


def test_few_attention_splits_walk_several_key_tiles_per_wave():
    _run("mini_hd128", [1500, 700, 90], 3, 66, splits=2)


def test_attention_work_list_with_very_different_lengths():
    # one to a dozen splits per sequence in the same launch (splits in proportion to the lengths)
    _run("step_hd128", [20, 300, 1500, 64, 700], 3, 75)


def test_long_batched_run_keeps_its_graph_while_the_sequences_grow():
    # 140 steps on one cached graph: every sequence crosses key-tile and page boundaries several times, so the splits
    # of the attention work list (fixed when the graph was built) get longer, and new pages enter the tables
    _run("step_hd128", [60, 130, 20], 140, 77)


def test_attention_without_a_work_list_when_the_batch_needs_too_many_items():
    # one KV head: the smallest splits still fit one round of the compute units, 7 x 17 items exceed the list
    _run("mini_hd128", [2048, 2040, 2000, 2048, 1990, 2030, 2010], 2, 76)


def test_other_page_size_uses_the_generic_attention_kernel():
    _run("mini_bf16", [70, 130, 45], 4, 68, page=32)


def test_degenerate_masks_in_one_batch():
    # one sequence skips every layer, one keeps every layer, one keeps a layer nobody else keeps
    # alone, and layer 2 is kept by nobody but the all-keep sequence
    masks = [[0, 0, 0, 0], [1, 1, 1, 1], [0, 1, 0, 0], [1, 0, 0, 1]]
    _run("mini_bf16", [16, 31, 48, 17], 5, 69, masks=masks)      # prompts end exactly at / next to page boundaries


def test_more_sequences_than_slots_run_in_groups():
    _run("mini_bf16", [18 + b for b in range(19)], 3, 67)        # 19 sequences: a group of 16 and one of 3


def test_shared_pass_agrees_with_one_pass_per_sequence():
    desc = CONFIGS["mini_bf16"]
    prompts = [make_prompt(desc.vocab, n, 70 + i) for i, n in enumerate((17, 64, 33, 40, 25))]
    masks = _masks(desc.n_layers, 5, 71)
    steps = [[3 + s, 40 + s, 900 + s, 11 + s, 1500 + s] for s in range(8)]
    outs = {}
    for path in (0, 1, 2):
        desc, w, router, ctx = build("mini_bf16", 71, max_batch=5, max_seq_len=128)
        ctx.set_option(OPT_BATCH_PATH, min(path, 1))
        ctx.set_option(9, 0 if path == 2 else 1)      # 2: shared pass over the caller's row-major matrices
        _prefill(ctx, desc, prompts)
        for b, m in enumerate(masks):
            ctx.set_mask(b, m)
        outs[path] = _decode(ctx, desc, steps, B=5)
        ctx.close()
    # same arithmetic up to the 16-bit split of the activations and the order of the sums
    assert float((outs[0][0] - outs[1][0]).abs().max()) <= 3e-3
    # tile-order copies or row-major matrices: the same products in the same order; with the tile-order kernels the
    # sum of squares behind 1/rms comes from the projections' epilogues, added in another order (2^-23 relative)
    scale = float(outs[2][0].abs().max())
    assert float((outs[1][0] - outs[2][0]).abs().max()) <= 2e-5 * scale and torch.equal(outs[1][1], outs[2][1])


def test_shared_pass_is_refused_for_fp32_models():
    import paper_2410_12513_amd as P
    desc, w, router, ctx = build("mini_fp32", 73, max_batch=2, max_seq_len=64)
    ctx.set_option(OPT_BATCH_PATH, 1)
    _prefill(ctx, desc, [make_prompt(desc.vocab, 20, 73), make_prompt(desc.vocab, 12, 74)])
    tin = torch.tensor([1, 2], dtype=torch.int32, device="cuda")
    with pytest.raises(P.FirstError) as e:
        ctx.decode_step(tin, None, tin)
    assert e.value.code == -2
    ctx.set_option(OPT_BATCH_PATH, -1)
    ctx.decode_step(tin, None, tin)
    ctx.close()
