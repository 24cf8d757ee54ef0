"""Checks that look at single kernels through the C ABI: the attention kernels' own probabilities
(blocked keys exactly 0), the cross-entropy kernel's workgroup sizes, Adam on a bf16 context at the
benchmark's module sizes, error paths of the boundary and non-default hyper-parameters."""
import dataclasses

import numpy as np
import pytest

import mm_synth
from oracle.mammoth_oracle import build_from_setup, module_layout
from paper_2403_07544_amd import MM_ENONFINITE, MM_ERANGE, MMError, Context
from tests.gpu_helpers import check_grads, check_touched, make_pair, say
from tests.helpers import tiny_batch, tiny_setup

pytestmark = pytest.mark.gpu

F32_TOL = dict(rel_tol=1e-4, cos_tol=0.9999999, floor_frac=1e-3)


# ------------------------------------------------------------------------------------------------
# attention probabilities read off the step's own forward attention kernel
# ------------------------------------------------------------------------------------------------
def _check_probs(ctx, orc, batch, H, tol_rel, tol_abs, label):
    B, S_max = batch.src_ids.shape
    U_max = batch.tgt_ids.shape[1] - 1
    s_len, u_len = batch.lengths[:, 0], batch.lengths[:, 1] - 1
    tr = orc.trace
    for kind, key, blocked, Lq, Lk, q_len in (("enc", "enc_P", tr["enc_blocked"], S_max, S_max, s_len),
                                              ("dec_self", "dec_self_P", tr["dec_blocked"], U_max, U_max, u_len),
                                              ("dec_cross", "dec_cross_P", tr["cross_blocked"], U_max, S_max, u_len)):
        for layer, P_ref in enumerate(tr[key]):
            P = ctx.mm_debug_attention(kind, layer, B, H).reshape(B, H, Lq, Lk).astype(np.float64)
            real_q = np.arange(Lq)[None, :] < q_len[:, None]                       # [B, Lq]
            blk = np.broadcast_to(np.asarray(blocked)[:, None, :, :], P.shape)
            rq = np.broadcast_to(real_q[:, None, :, None], P.shape)
            # a blocked key has probability exactly 0 in the kernel's output, bit for bit
            assert not P[blk & rq].any(), f"{label} {kind}[{layer}]: a blocked key has non-zero probability"
            # rows that do not exist (beyond the sentence) are never produced
            assert not P[~rq].any(), f"{label} {kind}[{layer}]: a padding query row was written"
            open_ = ~blk & rq
            ref = np.asarray(P_ref, dtype=np.float64)
            err = np.abs(P - ref)[open_]
            bound = (tol_rel * np.abs(ref) + tol_abs)[open_]
            assert (err <= bound).all(), f"{label} {kind}[{layer}]: probability off by {err.max():.3e}"
            # every open key keeps a positive probability (none is skipped by tile-level masking)
            assert (P[open_ & (ref > 20 * tol_abs)] > 0).all(), f"{label} {kind}[{layer}]: an open key got probability 0"
            sums = P.sum(axis=-1)[np.broadcast_to(real_q[:, None, :], (B, H, Lq))]
            assert np.abs(sums - 1).max() <= tol_rel * 4 + tol_abs * Lk, f"{label} {kind}[{layer}]: rows sum to {sums.min()}..{sums.max()}"
    say(f"  {label}: probabilities of {len(tr['enc_P'])} + 2 x {len(tr['dec_self_P'])} attention blocks match; blocked keys exactly 0")


def test_attention_kernel_probabilities_bf16_mfma():
    """bf16 context with 64-wide heads (the MFMA attention kernels): ragged sentences from one token to
    150, so that query tiles, several key tiles, the causal diagonal and the sentence end all occur."""
    setup = tiny_setup(d=128, H=2, F_=128, V=56, adapters=False, dtype="bf16", max_len=160)
    lengths = [(1, 2), (150, 149), (33, 65), (64, 33), (65, 2), (7, 130), (128, 129), (97, 31)]
    batch = tiny_batch(setup, lengths=lengths)
    say(f"[case] attention probabilities, bf16 MFMA kernels, {batch.n_src_tokens} src / {batch.n_tgt_tokens} tgt tokens")
    ctx, orc = make_pair(setup, keep_trace=True, max_batch_tokens=2048)
    ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    # probabilities leave the kernel rounded to bf16 (2^-9 relative); the queries and keys it reads are
    # bf16 products of bf16 activations, which moves a score by ~1e-2 relative
    _check_probs(ctx, orc, batch, 2, tol_rel=3e-2, tol_abs=2e-4, label="bf16")
    ctx.close()


def test_attention_kernel_probabilities_fp32():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapters=False, dtype="f32", max_len=40)
    batch = tiny_batch(setup, lengths=[(1, 2), (40, 39), (17, 33), (2, 2), (33, 17)])
    say("[case] attention probabilities, fp32 kernels")
    ctx, orc = make_pair(setup, keep_trace=True)
    ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    _check_probs(ctx, orc, batch, 2, tol_rel=1e-4, tol_abs=1e-7, label="fp32")
    ctx.close()


# ------------------------------------------------------------------------------------------------
# cross-entropy kernel: every workgroup size (64, 256, 1024 threads; register-resident rows)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,V", [("f32", 2048), ("f32", 16384), ("bf16", 4096), ("bf16", 16384)])
def test_cross_entropy_workgroup_sizes(dtype, V):
    """Vocabulary sizes that select the 256- and 1024-thread online-softmax kernel (several wavefronts
    share a row, and the row is overwritten with the gradient in the same kernel) and the smallest
    register-resident case."""
    setup = tiny_setup(d=32, H=2, F_=64, V=V, adapters=False, split_enc=False, enc_layers=(1, 0), dec_layers=1,
                       dtype=dtype, max_len=24)
    batch = tiny_batch(setup, lengths=((5, 4), (3, 7), (8, 2), (1, 5), (24, 25), (2, 2), (17, 9)))
    say(f"[case] cross-entropy at V={V}, {dtype}")
    ctx, orc = make_pair(setup)
    loss = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    ref = orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    say(f"  loss {loss:.6f} oracle {ref:.6f}")
    assert abs(loss - ref) <= (1e-4 if dtype == "f32" else 1e-2) * abs(ref)
    gen = orc.routes[0][-1]
    if dtype == "f32":
        check_grads(ctx, orc, orc.routes[0], label=f"V={V}", **F32_TOL)
    else:   # the generator's gradient is dz itself times h: its tensors see the loss kernel directly
        from tests.test_gpu_parity import SMALL_BF16_TOL
        check_grads(ctx, orc, [gen], label=f"V={V}", **SMALL_BF16_TOL)
    ctx.close()


# ------------------------------------------------------------------------------------------------
# hyper-parameters other than the defaults; error paths
# ------------------------------------------------------------------------------------------------
def _with_shape(setup, **kw):
    return dataclasses.replace(setup, shape=dataclasses.replace(setup.shape, **kw))


def test_no_label_smoothing_and_other_adam_constants():
    """label_smoothing = 0 (plain negative log-likelihood) and beta1/beta2/eps away from the defaults:
    step parity at the fp32 bar, then the update in isolation within 2 ulp."""
    setup = _with_shape(tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, dtype="f32", max_len=24),
                        label_smoothing=0.0, adam_beta1=0.8, adam_beta2=0.95, adam_eps=1e-6)
    say("[case] label_smoothing 0, Adam (0.8, 0.95, 1e-6)")
    ctx, orc = make_pair(setup)
    batch = tiny_batch(setup, lengths=((5, 4), (3, 7), (8, 2), (1, 5), (24, 25), (2, 2), (17, 9)))
    loss = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    ref = orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert abs(loss - ref) <= 1e-4 * abs(ref)
    check_grads(ctx, orc, orc.routes[0], label="eps_ls=0", **F32_TOL)
    # the update: first on the GPU's own gradient, then on a drawn one, against the fp32 oracle fed the same
    o32 = build_from_setup(setup, dtype=np.float32, perturbed=True, fill_params=mm_synth.fill_params)
    o32.b1, o32.b2, o32.adam_eps = (float(np.float32(x)) for x in (o32.b1, o32.b2, o32.adam_eps))
    rng = np.random.default_rng(11)
    for step in range(2):
        for j in orc.routes[0]:
            if step == 0:
                g = ctx.mm_get_grads(j)
            else:
                g = (rng.standard_normal(o32.modules[j].total) * 1e-3).astype(np.float32)
                ctx.mm_set_grads(j, g, 2)
            o32.modules[j].grad[:] = g
            o32.modules[j].touched = 1 + step
        ctx.mm_apply_update(None, 3e-3)
        o32.apply_update(None, 3e-3)
        for j in orc.routes[0]:
            gm, gv, t = ctx.mm_get_adam(j)
            for got, want, what in ((ctx.mm_get_params(j), o32.modules[j].theta, "theta"), (gm, o32.modules[j].m, "m"),
                                    (gv, o32.modules[j].v, "v")):
                ulp = np.spacing(np.abs(want).astype(np.float32))
                bad = np.abs(got.astype(np.float64) - want.astype(np.float64)) > 2 * ulp
                assert not bad.any(), (step, j, what, int(bad.sum()))
            assert t == step + 1
    ctx.close()


def test_non_finite_loss_is_reported():
    """A generator bias of +inf makes the loss non-finite: MM_ENONFINITE, use counts stand (the
    step's gradients have been added, as the header says), the next step on repaired weights works."""
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapters=False, dtype="f32", max_len=24)
    ctx, orc = make_pair(setup)
    batch = tiny_batch(setup)
    gen = orc.routes[0][-1]
    good = ctx.mm_get_params(gen)
    bad = good.copy()
    spec = {s.name: s for s in orc.modules[gen].specs}["bg"]
    bad[spec.offset + 5] = np.inf
    ctx.mm_set_params(gen, bad)
    with pytest.raises(MMError) as ei:
        ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert ei.value.status == MM_ENONFINITE
    assert all(ctx.mm_get_touched()[j] == 1 for j in orc.routes[0])
    with pytest.raises(MMError) as ei:
        ctx.mm_last_loss()
    assert ei.value.status == MM_ENONFINITE
    # the caller decides: here it discards the step by overwriting the buckets, repairs the weights and goes on
    for j in orc.routes[0]:
        ctx.mm_set_grads(j, np.zeros_like(ctx.mm_get_params(j)), 0)
    ctx.mm_set_params(gen, good)
    loss = ctx.mm_train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    ref = orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert abs(loss - ref) <= 1e-4 * abs(ref)
    check_grads(ctx, orc, orc.routes[0], label="after non-finite", **F32_TOL)
    ctx.close()


def _keep_gpu_busy():
    """Enqueues some tens of milliseconds of unrelated work on the stream the context uses (the
    default one), so that what the test enqueues next is still waiting when the host moves on."""
    import torch
    x = torch.ones(8192, 8192, device="cuda")
    for _ in range(6):
        x = (x @ x) * 1e-4
    return x


@pytest.mark.parametrize("step_still_running", [False, True])
def test_bad_device_ids_then_update_changes_nothing(step_still_running):
    bad_ids_then_update(step_still_running, "mm_apply_update")


def bad_ids_then_update(step_still_running, entry):
    """A step enqueued without waiting (out_loss NULL) whose device-resident ids are bad, followed
    by the update: the step had no effect, so no module may take an update - parameters, Adam state
    and step counts bit-unchanged, use counts as the oracle's - for all modules and for a subset.
    With step_still_running the GPU is kept busy, so the update is enqueued while the step has not
    run yet and the kernel itself has to take the outcome of the step into account."""
    import torch
    hold = _keep_gpu_busy if step_still_running else (lambda: None)
    setup = tiny_setup(d=32, H=2, F_=64, V=56, n_lang=3, adapter_dim=16, dtype="bf16", max_len=24)
    ctx, orc = make_pair(setup)
    apply_update = getattr(ctx, entry)
    names = [n for n, _ in setup.tasks]
    batch = tiny_batch(setup)
    t01, t21 = names.index("0-1"), names.index("2-1")
    # one good step of 2-1 first: the modules it shares with 0-1 have a count of 1 that must survive
    ctx.mm_train_step(t21, batch.src_ids, batch.tgt_ids, batch.lengths)
    orc.train_step(t21, batch.src_ids, batch.tgt_ids, batch.lengths)
    src = torch.tensor(batch.src_ids, dtype=torch.int32, device="cuda")
    tgt = torch.tensor(batch.tgt_ids, dtype=torch.int32, device="cuda")
    src[0, 0] = setup.shape.vocab + 3
    torch.cuda.synchronize()
    n_mod = len(orc.modules)
    before = {j: (ctx.mm_get_params(j), ctx.mm_get_working(j), *ctx.mm_get_adam(j)) for j in range(n_mod)}
    only_01 = [j for j in orc.routes[t01] if j not in orc.routes[t21]]
    assert len(only_01) >= 2

    def only_01_unchanged():
        for j in only_01:
            th, w, m, v, t = before[j]
            m2, v2, t2 = ctx.mm_get_adam(j)
            assert np.array_equal(th, ctx.mm_get_params(j)) and np.array_equal(w, ctx.mm_get_working(j)), j
            assert np.array_equal(m, m2) and np.array_equal(v, v2) and t == t2 == 0, j

    # part 1: update only modules that nothing but the bad step used
    hold()
    assert ctx.mm_train_step(t01, src, tgt, batch.lengths, sync=False) is None
    apply_update(only_01, 1e-3)
    with pytest.raises(MMError) as ei:
        ctx.mm_last_loss()
    assert ei.value.status == MM_ERANGE
    check_touched(ctx, orc)                 # the bad step is not counted; 2-1's modules still at one use
    only_01_unchanged()
    for j in orc.routes[t21]:
        assert ctx.mm_get_adam(j)[2] == 0
    # part 2: update everything: modules of the good step move once with n_j = 1, the others not at all
    hold()
    assert ctx.mm_train_step(t01, src, tgt, batch.lengths, sync=False) is None
    apply_update(None, 1e-3)
    with pytest.raises(MMError) as ei:
        ctx.mm_last_loss()
    assert ei.value.status == MM_ERANGE
    orc.apply_update(None, 1e-3)
    check_touched(ctx, orc)
    only_01_unchanged()
    for j in orc.routes[t21]:
        assert ctx.mm_get_adam(j)[2] == 1
        assert np.abs(ctx.mm_get_params(j) - orc.modules[j].theta).max() <= 2.5e-3
    # part 3: a good step of 0-1 and the update behind it, again without waiting in between
    hold()
    assert ctx.mm_train_step(t01, batch.src_ids, batch.tgt_ids, batch.lengths, sync=False) is None
    apply_update(None, 1e-3)
    orc.train_step(t01, batch.src_ids, batch.tgt_ids, batch.lengths)
    orc.apply_update(None, 1e-3)
    ctx.mm_last_loss()
    check_touched(ctx, orc)
    for j in range(n_mod):
        assert ctx.mm_get_adam(j)[2] == orc.modules[j].t, j
        assert np.abs(ctx.mm_get_params(j) - orc.modules[j].theta).max() <= 5e-3, j
    for j in only_01:
        assert not np.array_equal(before[j][0], ctx.mm_get_params(j)), j
    ctx.close()


# ------------------------------------------------------------------------------------------------
# Adam on a bf16 context at the benchmark's module sizes
# ------------------------------------------------------------------------------------------------
def test_adam_bf16_context_at_config2_module_sizes():
    """A decoder stack (25.2 M parameters: several thousand chunks, an odd tail) and an embedding
    table (16.4 M) of set-up 2's shape on a bf16 context: theta, m, v within 2 ulp of the fp32 oracle
    on the same gradient, the working copy the round-to-nearest-even bf16 of the new theta bit for
    bit, the table's bucket all zero afterwards (only the pieces that held a gradient are cleared)."""
    import torch
    sh = mm_synth.build_setup(2).shape
    ctx = Context(sh.d_model, sh.n_heads, sh.d_ff, sh.vocab, "bf16", sh.max_len, 4096)
    mods = [("dec", dict(position=0, n_layers=6, owns_final_norm=True)), ("tgt_emb", {})]
    rng = np.random.default_rng(5)
    b1, b2, eps = (float(np.float32(x)) for x in (0.9, 0.98, 1e-9))
    state = []
    for kind, kw in mods:
        j = ctx.mm_register_module(kind, "x", **kw)
        _, total = ctx.mm_get_layout(j)
        specs, total_ref = module_layout(kind, sh.d_model, sh.d_ff, sh.vocab, kw.get("n_layers", 0), kw.get("owns_final_norm", False))
        assert total == total_ref
        theta = (rng.standard_normal(total) * 0.02).astype(np.float32)
        ctx.mm_set_params(j, theta)
        state.append(dict(j=j, total=total, theta=theta, m=np.zeros(total, np.float32), v=np.zeros(total, np.float32), kind=kind))
    say(f"[case] Adam on a bf16 context: {[s['total'] for s in state]} parameters")
    lr = np.float32(2e-4)
    for step in range(2):
        for s in state:
            g = (rng.standard_normal(s["total"]) * 10.0 ** rng.integers(-6, 0, s["total"])).astype(np.float32)
            if s["kind"] == "tgt_emb":          # most rows of a table have no gradient in a step
                rows = g.reshape(sh.vocab, sh.d_model)
                rows[rng.random(sh.vocab) < 0.9] = 0
            n_uses = 1 + step
            ctx.mm_set_grads(s["j"], g, n_uses)
            s["g"], s["n"] = g, n_uses
        ctx.mm_apply_update(None, float(lr))
        t = step + 1
        for s in state:
            # the fp32 operation sequence of the update, one rounding per operation
            g = s["g"] / np.float32(s["n"])
            s["m"] = np.float32(b1) * s["m"] + np.float32(1 - np.float32(b1)) * g
            s["v"] = np.float32(b2) * s["v"] + np.float32(1 - np.float32(b2)) * g * g
            mh = s["m"] / np.float32(1 - b1 ** t)
            vh = s["v"] / np.float32(1 - b2 ** t)
            s["theta"] = s["theta"] - lr * mh / (np.sqrt(vh) + np.float32(eps))
            gm, gv, gt = ctx.mm_get_adam(s["j"])
            th = ctx.mm_get_params(s["j"])
            for got, want, what in ((th, s["theta"], "theta"), (gm, s["m"], "m"), (gv, s["v"], "v")):
                ulp = np.spacing(np.abs(want).astype(np.float32))
                bad = np.abs(got.astype(np.float64) - want.astype(np.float64)) > 2 * ulp
                assert not bad.any(), (step, s["kind"], what, int(bad.sum()))
            assert gt == t
            rne = torch.from_numpy(th).to(torch.bfloat16).to(torch.float32).numpy()
            assert np.array_equal(ctx.mm_get_working(s["j"]), rne), (step, s["kind"], "working copy")
            assert not ctx.mm_get_grads(s["j"]).any()
            if s["kind"] == "tgt_emb":
                assert not ctx.mm_get_bucket_memory(s["j"]).any(), "the table's bucket memory is not all zero after the update"
            s["theta"], s["m"], s["v"] = th, gm, gv          # go on from the GPU's state
    ctx.close()
