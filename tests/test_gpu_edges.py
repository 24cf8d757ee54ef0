"""Edge cases of the GPU path against the oracle: degenerate and maximal batch shapes, padding
width, long sentences (the 8-key-tile attention path), and limits set at context creation."""
import numpy as np
import pytest

import mm_synth
from tests.gpu_helpers import check_grads, check_integer_artefacts, check_touched, make_pair, say
from tests.helpers import tiny_batch, tiny_setup
from tests.test_gpu_parity import F32_TOL, bf16_tol

pytestmark = pytest.mark.gpu


def _run(setup, batch, dtype, task=0, max_batch_tokens=None, label=""):
    ctx, orc = make_pair(setup, keep_trace=True, max_batch_tokens=max_batch_tokens)
    loss = ctx.mm_train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    ref = orc.train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    say(f"  {label}: loss {loss:.6f} oracle {ref:.6f}")
    assert abs(loss - ref) <= (1e-4 if dtype == "f32" else 1e-2) * abs(ref)
    check_integer_artefacts(ctx, orc, batch, task)
    check_touched(ctx, orc)
    tol = F32_TOL if dtype == "f32" else bf16_tol(min(batch.n_src_tokens, batch.n_tgt_tokens))
    check_grads(ctx, orc, orc.routes[task], label=label, **tol)
    return ctx, orc


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_batches(dtype):
    d, H = (32, 2) if dtype == "f32" else (128, 2)
    setup = tiny_setup(d=d, H=H, F_=64, V=56, adapter_dim=16, dtype=dtype, max_len=24)
    for name, lengths in (("one pair, one token each way", ((1, 2),)),
                          ("all sentences of length one", ((1, 2),) * 5),
                          ("one long pair", ((24, 25),)),
                          ("long and short mixed", ((24, 2), (1, 25), (24, 25), (1, 2)))):
        say(f"[case] {dtype} {name}")
        _run(setup, tiny_batch(setup, lengths=lengths), dtype, label=name)


def test_padding_width_changes_nothing_bit_exactly():
    setup = tiny_setup(d=128, H=2, F_=64, V=56, adapter_dim=16, dtype="bf16", max_len=24)
    batch = tiny_batch(setup, lengths=((5, 4), (3, 7), (6, 2), (9, 11)))
    wide_src = np.pad(batch.src_ids, ((0, 0), (0, 24 - batch.src_ids.shape[1])))
    wide_tgt = np.pad(batch.tgt_ids, ((0, 0), (0, 25 - batch.tgt_ids.shape[1])))
    outs = []
    for src, tgt in ((batch.src_ids, batch.tgt_ids), (wide_src, wide_tgt)):
        ctx, _ = make_pair(setup)
        loss = ctx.mm_train_step(0, src, tgt, batch.lengths)
        outs.append((loss, [ctx.mm_get_grads(j) for j in ctx.mm_get_route(0)]))
    assert outs[0][0] == outs[1][0]
    for a, b in zip(outs[0][1], outs[1][1]):
        assert np.array_equal(a, b)


def test_long_sentences_use_all_key_tiles():
    """Sentences up to 200 tokens (the big set-up's limit): 7 key tiles of 32, ragged last tile."""
    setup = tiny_setup(d=128, H=2, F_=128, V=256, adapter_dim=16, dtype="bf16", max_len=200)
    batch = tiny_batch(setup, lengths=((200, 201), (129, 150), (97, 33), (161, 199), (1, 2), (64, 65)))
    say(f"[case] long sentences: {batch.n_src_tokens} src / {batch.n_tgt_tokens} tgt tokens")
    _run(setup, batch, "bf16", max_batch_tokens=1024, label="len<=200")


def test_limits_are_enforced_and_reached():
    from paper_2403_07544_amd import MMError, MM_ERANGE
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    # exactly max_batch_tokens source tokens and exactly max_len wide: accepted
    batch = tiny_batch(setup, lengths=((24, 9),) * 4)
    ctx, orc = make_pair(setup, max_batch_tokens=96)
    loss = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    ref = orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert abs(loss - ref) <= 1e-4 * abs(ref)
    over = tiny_batch(setup, lengths=((24, 9),) * 4 + ((1, 2),))
    with pytest.raises(MMError) as ei:
        ctx.mm_train_step(0, over.src_ids, over.tgt_ids, over.lengths)
    assert ei.value.status == MM_ERANGE
    check_touched(ctx, orc)            # the refused step counted nothing
    check_grads(ctx, orc, orc.routes[0], label="after refusal", **F32_TOL)


def test_update_of_listed_modules_only():
    """mm_apply_update(ids): listed touched modules step; the others keep bucket and count."""
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    ctx, orc = make_pair(setup)
    batch = tiny_batch(setup)
    ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    route = orc.routes[0]
    some, rest = route[:3], route[3:]
    keep = {j: ctx.mm_get_grads(j) for j in rest}
    ctx.mm_apply_update(some + [some[0]], 1e-3)          # a repeated id is applied once
    orc.apply_update(some, 1e-3)
    check_touched(ctx, orc)
    for j in some:
        assert ctx.mm_get_adam(j)[2] == 1 and not ctx.mm_get_grads(j).any()
        assert np.abs(ctx.mm_get_params(j) - orc.modules[j].theta).max() <= 2.5e-3
    for j in rest:
        assert ctx.mm_get_adam(j)[2] == 0 and np.array_equal(ctx.mm_get_grads(j), keep[j])


def test_nine_decoder_layers():
    """More decoder layers than one multi-product launch takes (eight): the key/value projections
    of the encoder output and their input-gradient products go out in two groups, and the
    encoder's closing LayerNorm backward adds nine parts."""
    setup = tiny_setup(d=128, H=2, F_=64, V=56, adapter_dim=16, dtype="bf16", max_len=24, dec_layers=9)
    batch = tiny_batch(setup, lengths=((5, 4), (3, 7), (8, 2), (1, 5), (24, 25), (2, 2), (17, 9)))
    say("[case] nine decoder layers")
    _run(setup, batch, "bf16", label="9 decoder layers")
