"""Pins for the oracle's beam search (`beam_decode`).  The paper names no search procedure; the
reading is the textbook beam over summed log-probabilities.  What fixes it here: beam 1 is the
(separately pinned) greedy search; a beam wide enough to hold every prefix is an exhaustive
search, checked against brute force over all sequences scored with the library transcription of
the model; the returned score is recomputed from that transcription; finished hypotheses are
carried and compete by score; ties go to the lower hypothesis, then the lower token."""
import itertools

import numpy as np

from oracle import mammoth_oracle as mo
from tests.helpers import sharpen, tiny_batch, tiny_oracle, tiny_setup, torch_reference_logits

LENGTHS = ((5, 4), (3, 7), (8, 2), (1, 5), (6, 3))


def _sources(setup, lengths=LENGTHS, seed=3):
    b = tiny_batch(setup, lengths, seed)
    return b.src_ids, b.lengths[:, 0].copy()


def _logp_rows(orc, task, src_row, tokens):
    """log softmax of the library transcription's logit rows after BOS + tokens (one row per position)."""
    z = np.asarray(torch_reference_logits(orc, task, src_row, [mo.BOS] + list(tokens)), dtype=np.float64)
    mx = z.max(axis=1, keepdims=True)
    return z - (mx + np.log(np.exp(z - mx).sum(axis=1, keepdims=True)))


def _sequence_score(orc, task, src_row, tokens):
    lp = _logp_rows(orc, task, src_row, tokens[:-1])
    return float(sum(lp[t, v] for t, v in enumerate(tokens)))


def test_beam_one_is_greedy_and_scores_are_sequence_log_probabilities():
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    src, s_len = _sources(setup)
    sharpen(orc, 6.0, 0.8)
    for task in range(len(orc.routes)):
        g_ids, g_n = orc.greedy_decode(task, src, s_len, 7)
        ids, n, score = orc.beam_decode(task, src, s_len, 7, 1)
        assert np.array_equal(ids, g_ids) and np.array_equal(n, g_n)
        for b in range(len(s_len)):
            ref = _sequence_score(orc, task, src[b, :s_len[b]], ids[b, :n[b]].tolist())
            assert abs(score[b] - ref) <= 1e-9 * max(1.0, abs(ref))


def test_wide_beam_is_exhaustive_search():
    """V = 8 and three tokens: 57 prefixes without EOS, so a beam of 64 never drops one and the
    result must be the best of all 400 complete sequences (brute force, library logits)."""
    setup = tiny_setup(V=8)
    src, s_len = _sources(setup, LENGTHS[:3])
    shapes = set()
    for scale, eos_shift in ((1.0, 0.0), (8.0, 0.5), (8.0, 2.0), (12.0, -1.0)):
        orc = tiny_oracle(setup)
        sharpen(orc, scale, eos_shift)
        ids, n, score = orc.beam_decode(0, src, s_len, 3, 64)
        for b in range(len(s_len)):
            row = src[b, :s_len[b]]
            best, best_seq = -np.inf, None
            open_prefixes = [()]
            for depth in range(3):
                nxt = []
                for pre in open_prefixes:
                    lp = _logp_rows(orc, 0, row, pre)
                    base = sum(lp[t, v] for t, v in enumerate(pre))
                    for v in range(8):
                        s = base + lp[len(pre), v]
                        seq = pre + (v,)
                        if v == mo.EOS or depth == 2:       # complete: ended, or as long as allowed
                            if s > best:
                                best, best_seq = s, seq
                        else:
                            nxt.append(seq)
                open_prefixes = nxt
            assert ids[b, :n[b]].tolist() == list(best_seq), (scale, eos_shift, b)
            assert abs(score[b] - best) <= 1e-9 * max(1.0, abs(best))
            shapes.add(int(n[b]))
    assert shapes >= {1, 3} or shapes >= {2, 3}, shapes    # early stops and full-length results both occur


def test_beam_scores_recompute_and_sentences_do_not_mix():
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    src, s_len = _sources(setup)
    sharpen(orc, 15.0, 1.5)      # some sentences end at once, others run to the limit
    ids, n, score = orc.beam_decode(1, src, s_len, 6, 3)
    assert ids.dtype == np.int32 and ids.shape == (len(s_len), 6)
    lens = set()
    for b in range(len(s_len)):
        toks = ids[b, :n[b]].tolist()
        assert (ids[b, n[b]:] == mo.PAD).all()
        assert mo.EOS not in toks[:-1]                      # nothing follows an EOS
        assert toks[-1] == mo.EOS or n[b] == 6
        ref = _sequence_score(orc, 1, src[b, :s_len[b]], toks)
        assert abs(score[b] - ref) <= 1e-9 * max(1.0, abs(ref))
        lens.add(int(n[b]))
        # one sentence alone gives the same result (hypotheses of different sentences never mix)
        one = orc.beam_decode(1, src[b:b + 1, :s_len[b]], s_len[b:b + 1], 6, 3)
        assert np.array_equal(one[0][0], ids[b]) and one[1][0] == n[b]
    assert len(lens) >= 2, lens


def test_finished_hypotheses_are_carried_and_ties_take_the_lowest_index():
    setup = tiny_setup()
    src, s_len = _sources(setup)
    B = len(s_len)
    # EOS far above everything: the best hypothesis is EOS alone, score ~ 0
    orc = tiny_oracle(setup)
    sharpen(orc, 1.0, 1e3)
    ids, n, score = orc.beam_decode(0, src, s_len, 5, 4)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (ids[:, 1:] == mo.PAD).all()
    assert (np.abs(score) < 1e-6).all()
    # EOS far below everything: every result has the full length
    orc = tiny_oracle(setup)
    sharpen(orc, 1.0, -1e3)
    ids, n, _ = orc.beam_decode(0, src, s_len, 5, 4)
    assert (n == 5).all() and (ids != mo.EOS).all()
    # equal logits everywhere: step one keeps tokens 0, 1 and 2 (= EOS, finished); in step two the
    # finished hypothesis (-ln V) beats every extension (-2 ln V) and is carried to the front
    orc = tiny_oracle(setup)
    gen = orc.modules[orc.parse_route(orc.routes[0])[4]]
    gen.p("Wg")[...] = 0
    gen.p("bg")[...] = 0
    ids, n, score = orc.beam_decode(0, src, s_len, 2, 3)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all()
    np.testing.assert_allclose(score, -np.log(orc.V), rtol=1e-12)
    # with a beam of two the finished one is not there (tokens 0 and 1 are kept): lowest ids win
    ids, n, score = orc.beam_decode(0, src, s_len, 2, 2)
    assert (n == 2).all() and (ids == 0).all()
    np.testing.assert_allclose(score, -2 * np.log(orc.V), rtol=1e-12)
    assert ids.shape == (B, 2)
