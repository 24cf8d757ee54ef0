"""Routed greedy translation on the GPU against the oracle (paper section 3.2: a task is
translated with its own modules).  Where two logits are closer than the arithmetic can tell
apart several outputs are correct, so a GPU output is checked for validity: fed back through the
oracle as decoder input, every produced token must be the oracle's row maximum up to a
tolerance, which also means that the first place a GPU sentence leaves the oracle's own output
is such a near-tie.  Structure (EOS, padding, counts) is exact."""
import numpy as np
import pytest

import mm_synth
from oracle import mammoth_oracle as mo
from tests.gpu_helpers import make_pair, say
from tests.helpers import sharpen, tiny_batch, tiny_setup

pytestmark = pytest.mark.gpu

# A logit row's error as a fraction of the row's spread (max - min).  fp32: rounding of a few
# hundred length-d sums, ~1e-6 relative, with margin.  bf16: every activation is rounded to 8
# significant bits (2^-9 relative) through up to a dozen residual blocks, and the logits
# themselves are stored in bf16: about 1e-2 of the spread; the worst seen is 2.6e-3 (full size).
TOL = {"f32": 2e-4, "bf16": 1e-2}
LENGTHS = ((5, 4), (3, 7), (8, 2), (1, 5), (6, 3), (2, 3), (7, 3), (4, 3), (24, 2), (13, 2))


def sharpened_pair(setup, scale, eos_shift):
    ctx, orc = make_pair(setup)
    sharpen(orc, scale, eos_shift)
    for j, m in enumerate(orc.modules):
        w = m.theta.astype(np.float32)
        m.theta[:] = w
        ctx.mm_set_params(j, w)
    return ctx, orc


def check_structure(ids, n, max_new):
    assert ids.dtype == np.int32 and n.dtype == np.int32 and ids.shape == (len(n), max_new)
    for b in range(len(n)):
        assert 1 <= n[b] <= max_new
        assert (ids[b, n[b]:] == mo.PAD).all()
        assert (ids[b, :n[b] - 1] != mo.EOS).all()
        if n[b] < max_new:
            assert ids[b, n[b] - 1] == mo.EOS


def check_valid(orc, task, src, s_len, ids, n, rel_tol, label=""):
    """Teacher-forced oracle logits of the GPU's own output: each token within rel_tol * spread
    of its row's maximum.  Returns the largest gap seen, as a fraction of the spread."""
    B, max_new = ids.shape
    dec_in = np.concatenate([np.full((B, 1), mo.BOS, dtype=np.int32), ids[:, :max_new - 1]], axis=1)
    z = orc.forward_logits(task, src, s_len, dec_in, n)
    worst = 0.0
    for b in range(B):
        for t in range(n[b]):
            row = z[b, t]
            gap = (row.max() - row[ids[b, t]]) / (row.max() - row.min())
            worst = max(worst, gap)
            assert gap <= rel_tol, f"{label}: sentence {b} step {t}: token {ids[b, t]} is {gap:.3e} of the spread below the maximum"
    return worst


def compare(ctx, orc, task, src, s_len, max_new, dtype, label):
    ids, n = ctx.mm_translate_greedy(task, src, s_len, max_new)
    check_structure(ids, n, max_new)
    worst = check_valid(orc, task, src, s_len, ids, n, TOL[dtype], label)
    ref_ids, ref_n = orc.greedy_decode(task, src, s_len, max_new)
    same = int((ids == ref_ids).all(axis=1).sum())
    say(f"  {label}: {same}/{len(n)} sentences identical to the oracle's, counts {n.tolist()}, worst gap {worst:.2e}")
    return ids, n, ref_ids, ref_n


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_translation_matches_oracle_on_small_models(dtype):
    d, scale, shift = (32, 6.0, 1.0) if dtype == "f32" else (128, 6.0, 2.0)
    setup = tiny_setup(d=d, H=2, F_=64, V=56, adapter_dim=16, dtype=dtype, max_len=24)
    ctx, orc = sharpened_pair(setup, scale, shift)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    for task in range(len(orc.routes)):
        say(f"[case] {dtype} task {task}: B={len(s_len)} max_new=12")
        ids, n, ref_ids, ref_n = compare(ctx, orc, task, src, s_len, 12, dtype, f"{dtype} task {task}")
        # the case is only worth something if sentences stop at different places and differ
        assert len(set(ref_n.tolist())) >= 4 and len({tuple(r) for r in ref_ids.tolist()}) >= 4
        if dtype == "f32":
            assert np.array_equal(ids, ref_ids) and np.array_equal(n, ref_n)
        else:
            assert (ids == ref_ids).all(axis=1).mean() >= 0.5
    ctx.close()


def test_translation_without_adapters_and_unsplit_stack():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapters=False, split_enc=False, dtype="f32", max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    say("[case] f32, no adapters, one-module stacks")
    ids, n, ref_ids, ref_n = compare(ctx, orc, 1, batch.src_ids, batch.lengths[:, 0].copy(), 9, "f32", "plain")
    assert np.array_equal(ids, ref_ids) and np.array_equal(n, ref_n)
    ctx.close()


def test_translation_with_head_size_32():
    """d = 64, two heads of 32 (the small-model cases use 16 and 64)."""
    setup = tiny_setup(d=64, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    say("[case] f32, head size 32")
    ids, n, ref_ids, ref_n = compare(ctx, orc, 0, batch.src_ids, batch.lengths[:, 0].copy(), 10, "f32", "dh=32")
    assert np.array_equal(ids, ref_ids) and np.array_equal(n, ref_n)
    ctx.close()


def test_translation_edge_shapes():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    for name, lengths, max_new in (("one sentence, one source token, one step", ((1, 2),), 1),
                                   ("one sentence up to the length limit", ((24, 2),), 24),
                                   ("many one-token sentences", ((1, 2),) * 7, 5),
                                   ("nine steps: the finished-check runs once mid-way", LENGTHS, 9),
                                   ("seventeen steps", LENGTHS[:3], 17)):
        say(f"[case] {name}")
        batch = tiny_batch(setup, lengths=lengths)
        ids, n, ref_ids, ref_n = compare(ctx, orc, 0, batch.src_ids, batch.lengths[:, 0].copy(), max_new, "f32", name)
        assert np.array_equal(ids, ref_ids) and np.array_equal(n, ref_n)
    # padding width of the source changes nothing
    batch = tiny_batch(setup, lengths=LENGTHS[:4])
    s_len = batch.lengths[:, 0].copy()
    a = ctx.mm_translate_greedy(0, batch.src_ids, s_len, 8)
    wide = np.pad(batch.src_ids, ((0, 0), (0, 24 - batch.src_ids.shape[1])))
    b = ctx.mm_translate_greedy(0, wide, s_len, 8)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # a shorter limit gives a prefix
    c = ctx.mm_translate_greedy(0, batch.src_ids, s_len, 3)
    assert np.array_equal(c[0], a[0][:, :3]) and np.array_equal(c[1], np.minimum(a[1], 3))
    ctx.close()


def test_forced_and_forbidden_eos_and_equal_logits():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    batch = tiny_batch(setup, lengths=LENGTHS[:5])
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    ctx, orc = sharpened_pair(setup, 1.0, 1e3)
    ids, n = ctx.mm_translate_greedy(0, src, s_len, 5)
    assert (n == 1).all() and (ids[:, 0] == mo.EOS).all() and (ids[:, 1:] == 0).all()
    ctx.close()
    ctx, orc = sharpened_pair(setup, 1.0, -1e3)
    ids, n = ctx.mm_translate_greedy(0, src, s_len, 5)
    assert (n == 5).all() and (ids != mo.EOS).all()
    ctx.close()
    ctx, orc = make_pair(setup)
    gen = orc.parse_route(orc.routes[0])[4]
    m = orc.modules[gen]
    m.p("Wg")[...] = 0
    m.p("bg")[...] = 0
    m.p("bg")[[9, 5]] = 2.5
    ctx.mm_set_params(gen, m.theta.astype(np.float32))
    ids, n = ctx.mm_translate_greedy(0, src, s_len, 3)
    assert (ids == 5).all() and (n == 3).all()          # the lower of two equal top logits
    ctx.close()


def test_translation_reads_device_ids_and_leaves_training_state_alone():
    import torch
    setup = tiny_setup(d=128, H=2, F_=64, V=56, adapter_dim=16, dtype="bf16", max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 2.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    host = ctx.mm_translate_greedy(1, src, s_len, 10)
    dev = ctx.mm_translate_greedy(1, torch.tensor(src, dtype=torch.int32, device="cuda"), s_len, 10)
    assert np.array_equal(host[0], dev[0]) and np.array_equal(host[1], dev[1])
    # a training step, a translation in between, then the same step again on a second context
    # that never translated: buckets, counts and parameters equal bit for bit
    ctx2, _ = sharpened_pair(setup, 6.0, 2.0)
    for c, translate in ((ctx, True), (ctx2, False)):
        c.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths, sync=False)
        if translate:
            c.mm_translate_greedy(1, src, s_len, 6)       # waits for the step in flight
        c.mm_train_step(1, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert np.array_equal(ctx.mm_get_touched(), ctx2.mm_get_touched())
    for j in range(ctx.mm_num_modules()):
        assert np.array_equal(ctx.mm_get_grads(j), ctx2.mm_get_grads(j))
        assert np.array_equal(ctx.mm_get_params(j), ctx2.mm_get_params(j))
    again = ctx.mm_translate_greedy(1, src, s_len, 10)
    assert np.array_equal(host[0], again[0])
    ctx.close(); ctx2.close()


def test_translation_refusals():
    from paper_2403_07544_amd import MMError, MM_EINVAL, MM_ERANGE
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24)
    ctx, _ = make_pair(setup, max_batch_tokens=64)
    batch = tiny_batch(setup, lengths=LENGTHS[:4])
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    bad_id = src.copy(); bad_id[0, 0] = 56
    late_id = src.copy(); late_id[1, -1] = 7
    zero_len = s_len.copy(); zero_len[2] = 0
    big = tiny_batch(setup, lengths=((24, 2),) * 3)
    for what, args, status in (("limit beyond max_len", (0, src, s_len, 25), MM_ERANGE),
                               ("no steps", (0, src, s_len, 0), MM_EINVAL),
                               ("unknown task", (99, src, s_len, 4), MM_EINVAL),
                               ("id outside the vocabulary", (0, bad_id, s_len, 4), MM_ERANGE),
                               ("id after the end", (0, late_id, s_len, 4), MM_ERANGE),
                               ("empty sentence", (0, src, zero_len, 4), MM_ERANGE),
                               ("too many source tokens", (0, big.src_ids, big.lengths[:, 0].copy(), 4), MM_ERANGE)):
        with pytest.raises(MMError) as ei:
            ctx.mm_translate_greedy(*args)
        assert ei.value.status == status, what
    ids, n = ctx.mm_translate_greedy(0, src, s_len, 4)       # still usable afterwards
    check_structure(ids, n, 4)
    ctx.close()


def test_config2_translation_at_full_size():
    """Transformer-base shape (512/8/2048, 6+6 layers, 32k vocabulary) in bf16: a batch of real
    length mix, outputs checked through the oracle's teacher-forced logits."""
    setup = mm_synth.build_setup(2)
    ctx, orc = sharpened_pair(setup, 4.0, 0.0)
    batch = mm_synth.make_batches(setup, 1)[0]
    B = 12
    s_len = batch.lengths[:B, 0].copy()
    src = np.ascontiguousarray(batch.src_ids[:B])
    say(f"[case] config 2 translation: B={B} source lengths {s_len.tolist()} max_new=10")
    ids, n = ctx.mm_translate_greedy(0, src, s_len, 10)
    check_structure(ids, n, 10)
    worst = check_valid(orc, 0, src, s_len, ids, n, TOL["bf16"], "config2")
    ref_ids, ref_n = orc.greedy_decode(0, src, s_len, 10)
    same = (ids == ref_ids).all(axis=1)
    say(f"  counts {n.tolist()}, {len({tuple(r) for r in ids.tolist()})} distinct outputs, worst gap {worst:.2e}, "
        f"{int(same.sum())}/{B} sentences identical to the oracle's")
    assert len({tuple(r) for r in ref_ids.tolist()}) >= 6      # the source decides the output
    assert same.mean() >= 0.75       # the others left it at a near-tie (checked above)
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_only_the_tasks_modules_are_read(dtype):
    """Section 3.2: a task needs only its own modules.  Every parameter of every module off the
    task's route is overwritten with NaN; translation and a training step of that task must give
    the same bits as before (one stray read of another module's memory would turn them into NaN)."""
    d = 32 if dtype == "f32" else 128
    setup = tiny_setup(d=d, H=2, F_=64, V=56, n_lang=3, adapter_dim=16, dtype=dtype, max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    task = 3
    route = set(ctx.mm_get_route(task))
    assert 0 < len(route) < ctx.mm_num_modules()
    before = ctx.mm_translate_greedy(task, src, s_len, 8)
    loss0 = ctx.mm_train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    grads0 = {j: ctx.mm_get_grads(j) for j in route}
    for j in range(ctx.mm_num_modules()):
        if j not in route:
            ctx.mm_set_params(j, np.full_like(ctx.mm_get_params(j), np.nan))
    after = ctx.mm_translate_greedy(task, src, s_len, 8)
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    for j in route:                                  # same step again from empty buckets
        ctx.mm_set_grads(j, np.zeros_like(grads0[j]), 0)
    loss1 = ctx.mm_train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert loss1 == loss0 and np.isfinite(loss1)
    for j in route:
        assert np.array_equal(ctx.mm_get_grads(j), grads0[j])
    ctx.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_a_context_holding_only_the_tasks_modules_translates_the_same(dtype):
    """Section 3.2 (inference): only the components a task needs have to be loaded.  A second
    context registers just the modules on one task's route, with the trained context's values,
    and must write the same tokens bit for bit; its memory is a fraction of the full model's."""
    from paper_2403_07544_amd import Context
    d = 32 if dtype == "f32" else 128
    setup = tiny_setup(d=d, H=2, F_=64, V=56, n_lang=3, adapter_dim=16, dtype=dtype, max_len=24)
    ctx, orc = sharpened_pair(setup, 6.0, 1.0)
    batch = tiny_batch(setup, lengths=LENGTHS)
    src, s_len = batch.src_ids, batch.lengths[:, 0].copy()
    task = 3
    route = ctx.mm_get_route(task)
    full = ctx.mm_translate_greedy(task, src, s_len, 8)
    sh = setup.shape
    small = Context(sh.d_model, sh.n_heads, sh.d_ff, sh.vocab, sh.dtype, sh.max_len, 256, sh.label_smoothing,
                    sh.adam_beta1, sh.adam_beta2, sh.adam_eps, sh.ln_eps)
    new_ids = []
    for j in route:
        ms = setup.modules[j]
        k = small.mm_register_module(ms.kind, ms.name, ms.position, ms.n_layers, ms.owns_final_norm,
                                     ms.adapter_dim, ms.stack)
        small.mm_set_params(k, ctx.mm_get_params(j))
        new_ids.append(k)
    t = small.mm_route_task(new_ids)
    assert small.mm_num_modules() == len(route) < ctx.mm_num_modules()
    part = small.mm_translate_greedy(t, src, s_len, 8)
    say(f"  {len(route)} of {ctx.mm_num_modules()} modules loaded; lengths {part[1].tolist()}")
    assert np.array_equal(full[0], part[0]) and np.array_equal(full[1], part[1])
    small.close()
    ctx.close()
