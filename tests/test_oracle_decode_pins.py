"""Pins for the oracle's routed inference (paper section 3.2: a task is translated with its own
modules only).  The logits are checked against the library transcription sentence by
sentence; the greedy loop against a loop written here over that transcription, against the
training step's own logits, and against the properties any greedy search has."""
import numpy as np
import pytest

from oracle import mammoth_oracle as mo
from tests.helpers import sharpen, tiny_batch, tiny_oracle, tiny_setup, torch_reference_logits

LENGTHS = ((5, 4), (3, 7), (8, 2), (1, 5), (6, 3), (2, 3), (7, 3), (4, 3))


def _sources(setup, lengths=LENGTHS, seed=3):
    b = tiny_batch(setup, lengths, seed)
    return b, b.src_ids, b.lengths[:, 0].copy()


def _library_greedy(orc, task, src_row, max_new):
    out = []
    for _ in range(max_new):
        z = torch_reference_logits(orc, task, src_row, [mo.BOS] + out)
        out.append(int(np.argmax(z[-1])))
        if out[-1] == mo.EOS:
            break
    return out


@pytest.mark.parametrize("adapters,split", [(True, True), (False, False)])
def test_forward_logits_against_library_transcription(adapters, split):
    setup = tiny_setup(adapters=adapters, split_enc=split)
    orc = tiny_oracle(setup)
    batch, src, s_len = _sources(setup)
    dec_in, dec_len = batch.tgt_ids[:, :-1], batch.lengths[:, 1] - 1
    for task in range(len(orc.routes)):
        z = orc.forward_logits(task, src, s_len, dec_in, dec_len)
        assert z.shape == (len(s_len), dec_in.shape[1], orc.V)
        for b in range(len(s_len)):
            ref = torch_reference_logits(orc, task, src[b, :s_len[b]], dec_in[b, :dec_len[b]])
            np.testing.assert_allclose(z[b, :dec_len[b]], ref, rtol=0, atol=1e-11)


def test_forward_logits_equal_training_step_logits():
    setup = tiny_setup()
    orc = tiny_oracle(setup, keep_trace=True)
    batch, src, s_len = _sources(setup)
    z = orc.forward_logits(1, src, s_len, batch.tgt_ids[:, :-1], batch.lengths[:, 1] - 1)
    orc.train_step(1, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert np.array_equal(z[orc.trace["dec_real"]], orc.trace["logits"])


def test_forward_logits_touch_no_bookkeeping():
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    batch, src, s_len = _sources(setup)
    before = [(m.theta.copy(), m.grad.copy(), m.touched) for m in orc.modules]
    orc.greedy_decode(0, src, s_len, 3)
    for m, (th, g, n) in zip(orc.modules, before):
        assert np.array_equal(m.theta, th) and np.array_equal(m.grad, g) and m.touched == n


@pytest.mark.parametrize("scale,eos_shift", [(1.0, 0.0), (5.0, 1.0), (7.0, 0.8)])
def test_greedy_against_loop_over_library_logits(scale, eos_shift):
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    _, src, s_len = _sources(setup)
    sharpen(orc, scale, eos_shift)
    max_new = 9
    n_seen = set()
    for task in range(len(orc.routes)):
        ids, n_out = orc.greedy_decode(task, src, s_len, max_new)
        for b in range(len(s_len)):
            ref = _library_greedy(orc, task, src[b, :s_len[b]], max_new)
            assert n_out[b] == len(ref)
            assert ids[b, :n_out[b]].tolist() == ref
            assert (ids[b, n_out[b]:] == mo.PAD).all()
            n_seen.add(int(n_out[b]))
    if eos_shift:
        # the shifted set-up is there to stop sentences at different places, mid-way included
        assert len([n for n in n_seen if 1 < n < max_new]) >= 3, n_seen


def test_greedy_tokens_are_row_maxima_of_teacher_forced_logits():
    """Feeding the produced tokens back as decoder input, each one is the arg-max of the logit
    row before it (computed through the training step's forward pass)."""
    setup = tiny_setup()
    orc = tiny_oracle(setup, keep_trace=True)
    _, src, s_len = _sources(setup)
    sharpen(orc, 7.0, 0.8)
    max_new = 7
    ids, n_out = orc.greedy_decode(0, src, s_len, max_new)
    B = len(s_len)
    tgt = np.zeros((B, max_new + 1), dtype=np.int32)
    tgt[:, 0] = mo.BOS
    tgt[:, 1:] = ids
    lengths = np.stack([s_len, n_out + 1], axis=1).astype(np.int32)
    orc.train_step(0, src, tgt, lengths)
    z = orc.trace["logits"]
    rows = np.concatenate([ids[b, :n_out[b]] for b in range(B)])
    assert np.array_equal(np.argmax(z, axis=1), rows)


def test_greedy_prefix_and_batch_independence():
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    _, src, s_len = _sources(setup)
    sharpen(orc, 7.0, 0.8)
    short, n_short = orc.greedy_decode(0, src, s_len, 4)
    long_, n_long = orc.greedy_decode(0, src, s_len, 7)
    assert len({tuple(r) for r in long_.tolist()}) >= 5     # the source decides the output
    assert np.array_equal(long_[:, :4], short)
    assert np.array_equal(np.minimum(n_long, 4), n_short)
    for b in range(len(s_len)):
        one, n_one = orc.greedy_decode(0, src[b:b + 1, :s_len[b]], s_len[b:b + 1], 7)
        assert np.array_equal(one[0], long_[b]) and n_one[0] == n_long[b]


def test_greedy_stopping_rules_and_lowest_index_on_ties():
    setup = tiny_setup()
    _, src, s_len = _sources(setup)
    B = len(s_len)
    # EOS far above everything: every sentence is just EOS
    orc = tiny_oracle(setup)
    sharpen(orc, 1.0, 1e3)
    ids, n = orc.greedy_decode(0, src, s_len, 5)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (ids[:, 1:] == mo.PAD).all()
    # EOS far below everything: never stops before the limit
    orc = tiny_oracle(setup)
    sharpen(orc, 1.0, -1e3)
    ids, n = orc.greedy_decode(0, src, s_len, 5)
    assert (n == 5).all() and (ids != mo.EOS).all()
    # all logits fixed by the bias, two of them equal on top: the lower index is taken
    orc = tiny_oracle(setup)
    gen = orc.modules[orc.parse_route(orc.routes[0])[4]]
    gen.p("Wg")[...] = 0
    gen.p("bg")[...] = 0
    gen.p("bg")[[9, 5]] = 2.5
    ids, n = orc.greedy_decode(0, src, s_len, 3)
    assert (ids == 5).all() and (n == 3).all()
    assert ids.dtype == np.int32 and ids.shape == (B, 3)
