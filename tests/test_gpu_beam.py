"""Routed beam search on the GPU against the oracle's `beam_decode` (the paper names no search
procedure; both sides implement the textbook beam over summed log-probabilities).  Scores are
fp32 on the GPU and fp64 in the oracle: where two candidates are closer than that arithmetic can
tell apart the beams may part ways, so a sentence that differs from the oracle's is checked for
validity instead: its reported score is the true log-probability of the sequence it reports, and
that log-probability is no worse than the oracle's best hypothesis by more than the tolerance.
Integer rules (carried finished hypotheses, tie order, padding, counts) are exact."""
import numpy as np
import pytest

import mm_synth
from oracle import mammoth_oracle as mo
from paper_2403_07544_amd import MM_EINVAL, MM_ERANGE, MMError
from tests.gpu_helpers import make_pair, say
from tests.helpers import tiny_batch, tiny_setup
from tests.test_gpu_translate import LENGTHS, check_structure, sharpened_pair

pytestmark = pytest.mark.gpu

# absolute error of a summed log-probability per produced token: logits to ~2e-4 (fp32) / ~1e-2
# (bf16) of their spread (see test_gpu_translate.TOL), spread here <= ~20
SCORE_TOL = {"f32": 5e-3, "bf16": 0.25}


def true_score(orc, task, src_row, toks):
    """log-probability of BOS -> toks under the oracle's model (fp64)."""
    dec_in = np.array([[mo.BOS] + list(toks[:-1])], dtype=np.int32)
    z = orc.forward_logits(task, src_row[None, :], np.array([len(src_row)], dtype=np.int32), dec_in,
                           np.array([len(toks)], dtype=np.int32))[0].astype(np.float64)
    mx = z.max(axis=1, keepdims=True)
    logp = z - (mx + np.log(np.exp(z - mx).sum(axis=1, keepdims=True)))
    return float(sum(logp[t, v] for t, v in enumerate(toks)))


def compare_beam(ctx, orc, task, src, s_len, max_new, beam, dtype, label, need_same=0.75):
    ids, n, score = ctx.mm_translate_beam(task, src, s_len, max_new, beam)
    check_structure(ids, n, max_new)
    assert score.dtype == np.float32 and score.shape == (len(n),)
    ref_ids, ref_n, ref_score = orc.beam_decode(task, src, s_len, max_new, beam)
    same = 0
    for b in range(len(n)):
        tol = SCORE_TOL[dtype] * n[b]
        mine = true_score(orc, task, src[b, :s_len[b]], ids[b, :n[b]].tolist())
        assert abs(score[b] - mine) <= tol, f"{label}: sentence {b}: reported {score[b]}, its sequence scores {mine}"
        if np.array_equal(ids[b], ref_ids[b]):
            same += 1
            assert n[b] == ref_n[b] and abs(score[b] - ref_score[b]) <= tol
        else:
            # the beams parted at a near-tie: the GPU's hypothesis must still be as good as the oracle's
            # best within the arithmetic's resolution (a self-consistent but worse hypothesis fails here)
            worst_len = max(int(n[b]), int(ref_n[b]))
            assert mine >= ref_score[b] - SCORE_TOL[dtype] * worst_len, \
                f"{label}: sentence {b}: its sequence scores {mine}, the oracle's best {ref_score[b]}"
    say(f"  {label}: beam {beam}: {same}/{len(n)} sentences identical to the oracle's, counts {n.tolist()}")
    assert same >= need_same * len(n), f"{label}: only {same} of {len(n)} sentences agree with the oracle"
    return ids, n, score, ref_ids


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_beam_search_matches_oracle_on_small_models(dtype):
    d = 32 if dtype == "f32" else 128
    setup = tiny_setup(d=d, H=2, F_=64, V=56, n_lang=3, adapter_dim=16, dtype=dtype, max_len=24)
    say(f"[case] beam search, small model, dtype={dtype}")
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    seen = set()
    for (scale, eos_shift), task, beam, max_new in (((15.0, 1.5), 1, 3, 6), ((6.0, 0.8), 0, 4, 9), ((8.0, 0.0), 4, 2, 5),
                                                    ((10.0, 1.0), 2, 8, 7)):
        ctx, orc = sharpened_pair(setup, scale, eos_shift)
        ids, n, score, ref_ids = compare_beam(ctx, orc, task, src, s_len, max_new, beam, dtype, f"task {task}")
        g_ids, _ = ctx.mm_translate_greedy(task, src, s_len, max_new)
        seen.add(bool((ids != g_ids).any()))
        ctx.close()
    assert True in seen          # somewhere the beam found something the greedy search did not


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_beam_of_one_is_the_greedy_search(dtype):
    d = 32 if dtype == "f32" else 128
    setup = tiny_setup(d=d, H=2, F_=64, V=56, adapter_dim=16, dtype=dtype, max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    for task in range(2):
        g_ids, g_n = ctx.mm_translate_greedy(task, src, s_len, 9)
        ids, n, score = ctx.mm_translate_beam(task, src, s_len, 9, 1)
        assert np.array_equal(ids, g_ids) and np.array_equal(n, g_n)
        assert np.isfinite(score).all() and (score <= 0).all()
    ctx.close()


def test_carried_hypotheses_tie_order_and_edge_shapes():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    B = len(s_len)
    # equal logits everywhere (decided by the integer rules alone): with three hypotheses the
    # finished one (EOS, -ln V) is carried past every extension (-2 ln V); with two it is not in
    # the beam and the lowest ids win
    ctx, orc = make_pair(setup)
    gen_id = orc.parse_route(orc.routes[0])[4]
    zeros = np.zeros_like(ctx.mm_get_params(gen_id))
    ctx.mm_set_params(gen_id, zeros)
    ids, n, score = ctx.mm_translate_beam(0, src, s_len, 2, 3)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (ids[:, 1] == mo.PAD).all()
    np.testing.assert_allclose(score, -np.log(56.0), rtol=1e-5)
    ids, n, score = ctx.mm_translate_beam(0, src, s_len, 2, 2)
    assert (n == 2).all() and (ids == 0).all()
    np.testing.assert_allclose(score, -2 * np.log(56.0), rtol=1e-5)
    ctx.close()
    # forced and forbidden EOS
    ctx, orc = sharpened_pair(setup, 1.0, 1e3)
    ids, n, score = ctx.mm_translate_beam(0, src, s_len, 5, 4)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (np.abs(score) < 1e-3).all()
    # a longer limit: every beam is finished after two steps, the host notices at its first look
    # (step 8) and stops; the history it walks back is shorter than max_new
    ids, n, score = ctx.mm_translate_beam(0, src, s_len, 20, 4)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (ids[:, 1:] == mo.PAD).all()
    assert (np.abs(score) < 1e-3).all()
    ctx.close()
    ctx, orc = sharpened_pair(setup, 1.0, -1e3)
    ids, n, _ = ctx.mm_translate_beam(0, src, s_len, 5, 4)
    assert (n == 5).all() and (ids != mo.EOS).all()
    ctx.close()
    # one sentence, the widest beam, one token; one-token source; as many tokens as max_len allows
    ctx, orc = sharpened_pair(setup, 8.0, 0.5)
    compare_beam(ctx, orc, 0, src[:1, :s_len[0]], s_len[:1], 1, 8, "f32", "one token")
    one = tiny_batch(setup, lengths=((1, 2),))
    compare_beam(ctx, orc, 1, one.src_ids, one.lengths[:, 0].copy(), 6, 3, "f32", "one-token source")
    compare_beam(ctx, orc, 0, src[:3], s_len[:3], 24, 2, "f32", "max_len tokens")
    ctx.close()


def test_beam_refusals_and_untouched_training_state():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 0.8)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    for beam in (0, -1, 9):
        with pytest.raises(MMError) as ei:
            ctx.mm_translate_beam(0, src, s_len, 4, beam)
        assert ei.value.status == MM_EINVAL
    with pytest.raises(MMError) as ei:
        ctx.mm_translate_beam(0, src, s_len, 25, 2)            # more tokens than max_len
    assert ei.value.status == MM_ERANGE
    with pytest.raises(MMError) as ei:
        ctx.mm_translate_beam(7, src, s_len, 4, 2)
    assert ei.value.status == MM_EINVAL
    # a step, a beam search, the same step again from the same state: same bits; nothing counted
    loss0 = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    route = ctx.mm_get_route(0)
    grads0 = {j: ctx.mm_get_grads(j) for j in route}
    touched0 = ctx.mm_get_touched().copy()
    import torch
    dev_src = torch.tensor(src, dtype=torch.int32, device="cuda")
    a = ctx.mm_translate_beam(0, dev_src, s_len, 6, 3)           # ids resident on the device
    b = ctx.mm_translate_beam(0, src, s_len, 6, 3)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert np.array_equal(ctx.mm_get_touched(), touched0)
    for j in route:
        assert np.array_equal(ctx.mm_get_grads(j), grads0[j])
    ctx.close()


def test_config2_beam_search_at_full_size():
    """Set-up 2's model and one of its batches (75 sentences x 4 hypotheses = 300 decoder rows):
    beam 1 equals the greedy search; with beam 4 a sample of sentences is compared with the
    oracle, and every sentence's reported score with the true log-probability of its sequence
    on that sample."""
    setup = mm_synth.build_setup(2)
    say("[case] set-up 2, beam search at full size")
    ctx, orc = sharpened_pair(setup, 4.0, 0.0)      # (as in the greedy search's full-size test)
    batch = mm_synth.make_batches(setup, 1)[0]
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    B = len(s_len)
    g_ids, g_n = ctx.mm_translate_greedy(0, src, s_len, 6)
    ids1, n1, _ = ctx.mm_translate_beam(0, src, s_len, 6, 1)
    agree = int((ids1 == g_ids).all(axis=1).sum())
    say(f"  beam 1 against greedy: {agree}/{B} identical")
    assert agree >= B - 2          # (a rounding tie between two logits after subtracting the row's lse may differ)
    ids, n, score = ctx.mm_translate_beam(0, src, s_len, 6, 4)
    check_structure(ids, n, 6)
    sample = [0, B // 2, B - 1]
    same = 0
    for b in sample:
        row = src[b, :s_len[b]]
        mine = true_score(orc, 0, row, ids[b, :n[b]].tolist())
        assert abs(score[b] - mine) <= SCORE_TOL["bf16"] * n[b], (b, score[b], mine)
        r_ids, r_n, r_score = orc.beam_decode(0, src[b:b + 1, :s_len[b]], s_len[b:b + 1], 6, 4)
        if np.array_equal(r_ids[0], ids[b]):
            same += 1
        else:                      # a near-tie sent the beams different ways: the GPU's is no worse than tolerance
            assert mine >= r_score[0] - SCORE_TOL["bf16"] * 6, (b, mine, r_score[0])
    say(f"  beam 4: {same}/{len(sample)} sampled sentences identical to the oracle's; counts {n[:8].tolist()}...")
    ctx.close()
