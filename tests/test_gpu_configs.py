"""Full-size parity: the benchmark set-ups at their real shapes, in the launch configuration
bench.py times, against the fp64 CPU oracle on the same seeded batch."""
import time

import numpy as np
import pytest

import mm_synth
from tests.gpu_helpers import check_grads, check_integer_artefacts, check_touched, make_pair, say
from tests.test_gpu_parity import BF16_TOL

pytestmark = pytest.mark.gpu


def test_config2_transformer_base_full_step():
    setup = mm_synth.build_setup(2)
    batch = mm_synth.make_batches(setup, 1)[0]
    say(f"[case] config 2 full size: B={len(batch.lengths)} S={batch.n_src_tokens} U={batch.n_tgt_tokens}")
    t0 = time.time()
    ctx, orc = make_pair(setup, perturbed=False)
    say(f"  built in {time.time() - t0:.1f}s")
    loss = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    say(f"  gpu loss {loss:.6f}")
    t0 = time.time()
    ref = orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    say(f"  oracle loss {ref:.6f} in {time.time() - t0:.1f}s")
    assert abs(loss - ref) <= 1e-2 * abs(ref)
    assert abs(ref - np.log(setup.shape.vocab)) < 0.2
    check_integer_artefacts(ctx, orc, batch, 0)
    check_touched(ctx, orc)
    worst = check_grads(ctx, orc, orc.routes[0], label="config2", **BF16_TOL)
    say(f"  worst tensor {worst}")
    lr = setup.shape.lr
    before = [ctx.mm_get_params(j) for j in orc.routes[0]]
    ctx.mm_apply_update(None, lr)
    for j, th0 in zip(orc.routes[0], before):
        th1 = ctx.mm_get_params(j)
        delta = np.abs(th1 - th0)
        assert delta.max() <= lr * 1.0001 + 1e-7          # first Adam step moves each weight by <= lr
        g = orc.modules[j].grad
        big = np.abs(g) > 1e-2 * np.abs(g).max()
        agree = np.sign(th0[big] - th1[big]) == np.sign(g[big])                # moves against the gradient
        assert agree.mean() > 0.999
        assert not ctx.mm_get_grads(j).any()
        w = ctx.mm_get_working(j)
        assert np.abs(w - th1).max() <= np.abs(th1).max() * 2.0 ** -8
    assert ctx.mm_get_touched().sum() == 0
