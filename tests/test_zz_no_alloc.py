"""mm_apply_update_noalloc (the update for callers that cannot allocate) against mm_apply_update:
same gradients in, bit-identical parameters, Adam state, working copies and counts out - on two
calls in a row, the second over fewer modules - and the limit on modules per call."""
import numpy as np
import pytest

import mm_synth
from paper_2403_07544_amd import MM_ERANGE, MMError, Context, context_from_setup
from tests.gpu_helpers import say
from tests.helpers import tiny_setup

pytestmark = pytest.mark.gpu


def _pair_of_contexts(setup):
    return [context_from_setup(setup, fill_params=mm_synth.fill_params, perturbed=True) for _ in range(2)]


def _same_state(a, b, modules):
    for j in modules:
        assert np.array_equal(a.mm_get_params(j), b.mm_get_params(j)), f"module {j}: parameters differ"
        assert np.array_equal(a.mm_get_working(j), b.mm_get_working(j)), f"module {j}: working copies differ"
        ma, va, ta = a.mm_get_adam(j)
        mb, vb, tb = b.mm_get_adam(j)
        assert np.array_equal(ma, mb) and np.array_equal(va, vb) and ta == tb, f"module {j}: Adam state differs"
        assert np.array_equal(a.mm_get_bucket_memory(j), b.mm_get_bucket_memory(j)), f"module {j}: buckets differ"
    assert np.array_equal(a.mm_get_touched(), b.mm_get_touched())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noalloc_update_equals_the_allocating_one(dtype):
    setup = tiny_setup(d=32, H=2, F_=64, V=56, n_lang=3, adapter_dim=16, dtype=dtype, max_len=24)
    ref, new = _pair_of_contexts(setup)
    n_mod = ref.mm_num_modules()
    say(f"[case] update without allocation, {dtype}, {n_mod} modules")
    rng = np.random.default_rng(2)
    sizes = [ref.mm_get_layout(j)[1] for j in range(n_mod)]

    def give(modules, uses):
        for j in modules:
            g = (rng.standard_normal(sizes[j]) * 10.0 ** rng.integers(-5, 0)).astype(np.float32)
            g[rng.random(sizes[j]) < 0.2] = 0
            for c in (ref, new):
                c.mm_set_grads(j, g, uses)

    # first call: every module; second call: a smaller set (the static table keeps the first call's entries)
    give(range(n_mod), 2)
    ref.mm_apply_update(None, 1e-3)
    new.mm_apply_update_noalloc(None, 1e-3)
    _same_state(ref, new, range(n_mod))
    assert all(new.mm_get_adam(j)[2] == 1 for j in range(n_mod))
    few = [n_mod - 1, 3, 0]
    give(few, 1)
    give([5], 3)                                   # has a gradient but is not asked for: must stay as it is
    ref.mm_apply_update(few, 2e-3)
    new.mm_apply_update_noalloc(few, 2e-3)
    _same_state(ref, new, range(n_mod))
    assert [new.mm_get_adam(j)[2] for j in few] == [2, 2, 2] and new.mm_get_adam(5)[2] == 1
    assert new.mm_get_touched()[5] == 3
    # modules without a use: a call that selects nothing touches nothing
    new.mm_apply_update_noalloc([1, 2], 1e-3)
    _same_state(ref, new, range(n_mod))
    for c in (ref, new):
        c.close()


def test_noalloc_update_refuses_more_modules_than_its_table_holds():
    ctx = Context(16, 1, 16, 56, "f32", 8, 64)
    n = 260
    ids = [ctx.mm_register_module("adapter", f"a{k}", n_layers=1, adapter_dim=16, stack="enc") for k in range(n)]
    size = ctx.mm_get_layout(ids[0])[1]
    g = np.full(size, 1e-3, dtype=np.float32)
    for j in ids:
        ctx.mm_set_grads(j, g, 1)
    before = ctx.mm_get_params(ids[7])
    with pytest.raises(MMError) as ei:
        ctx.mm_apply_update_noalloc(None, 1e-3)
    assert ei.value.status == MM_ERANGE and "256" in str(ei.value)
    assert ctx.mm_get_touched().tolist() == [1] * n and np.array_equal(before, ctx.mm_get_params(ids[7]))
    ctx.mm_apply_update_noalloc(ids[:256], 1e-3)          # exactly the limit works
    assert ctx.mm_get_touched().tolist() == [0] * 256 + [1] * 4
    assert ctx.mm_get_adam(ids[255])[2] == 1 and ctx.mm_get_adam(ids[256])[2] == 0
    ctx.close()


@pytest.mark.parametrize("step_still_running", [False, True])
def test_noalloc_update_behind_a_step_with_bad_ids(step_still_running):
    """The same sequence as the allocating entry point's test: a step with bad device-resident ids,
    enqueued without waiting, then the update - also while the step has not run yet."""
    from tests.test_gpu_hooks import bad_ids_then_update
    bad_ids_then_update(step_still_running, "mm_apply_update_noalloc")
