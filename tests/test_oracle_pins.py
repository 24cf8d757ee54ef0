"""Pins for the CPU oracle: everything here checks the oracle against something that is not
the oracle - finite differences, a library-autograd transcription, closed forms, brute force
and structural identities that follow from the paper's routing rules (section 3.2, Alg. 1)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import mm_synth
from oracle import mammoth_oracle as mo
from tests.helpers import (rel_l2, tiny_batch, tiny_oracle, tiny_setup, torch_reference_step)


def _loss_only(orc, task, batch):
    """Loss at the current parameters without disturbing buckets or counters."""
    saved = [(m.grad.copy(), m.touched) for m in orc.modules]
    loss = orc.train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    for m, (g, n) in zip(orc.modules, saved):
        m.grad[:] = g
        m.touched = n
    return loss


# ------------------------------------------------------------------------------------------
# 1. finite differences: every tensor of every used module, direction + single coordinates
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("task", [0, 1])
def test_finite_differences_every_tensor(task):
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    batch = tiny_batch(setup)
    orc.train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
    rng = np.random.default_rng(5)
    h = 1e-5
    worst = 0.0
    for j in orc.routes[task]:
        m = orc.modules[j]
        for s in m.specs:
            g = m.grad[s.offset:s.offset + s.size].copy()
            v = rng.standard_normal(s.size)
            v /= np.linalg.norm(v)
            th = m.theta[s.offset:s.offset + s.size]
            keep = th.copy()
            th[:] = keep + h * v
            lp = _loss_only(orc, task, batch)
            th[:] = keep - h * v
            lm = _loss_only(orc, task, batch)
            th[:] = keep
            fd = (lp - lm) / (2 * h)
            an = float(g @ v)
            # the difference quotient carries ~1e-16 * L / h ~ 5e-11 of rounding noise
            assert abs(fd - an) <= 2e-6 * abs(an) + 3e-10, (m.kind, s.name, fd, an)
            if abs(an) > 1e-4:
                worst = max(worst, abs(fd - an) / abs(an))
    assert 0 < worst < 2e-6


def test_finite_differences_single_coordinates_sign():
    """The bucket holds +dL/dtheta (the descent sign lives in the optimiser)."""
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    batch = tiny_batch(setup)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    rng = np.random.default_rng(11)
    for j in orc.routes[0]:
        m = orc.modules[j]
        nz = np.flatnonzero(np.abs(m.grad) > 1e-6)
        for idx in rng.choice(nz, size=min(4, len(nz)), replace=False):
            keep = m.theta[idx]
            m.theta[idx] = keep + 1e-5
            lp = _loss_only(orc, 0, batch)
            m.theta[idx] = keep - 1e-5
            lm = _loss_only(orc, 0, batch)
            m.theta[idx] = keep
            fd = (lp - lm) / 2e-5
            assert abs(fd - m.grad[idx]) <= 2e-6 * max(abs(fd), 1e-4), (m.kind, idx)
            assert np.sign(fd) == np.sign(m.grad[idx])


def test_fp32_oracle_close_to_fp64_oracle():
    setup = tiny_setup()
    o64, o32 = tiny_oracle(setup), tiny_oracle(setup, dtype=np.float32)
    batch = tiny_batch(setup)
    l64 = o64.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    l32 = o32.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert abs(l64 - l32) < 1e-5 * abs(l64)
    for j in o64.routes[0]:
        for s in o64.modules[j].specs:
            ref = o64.modules[j].g(s.name)
            if np.linalg.norm(ref) < 1e-9:      # exactly-zero gradients (key bias)
                assert np.abs(o32.modules[j].g(s.name)).max() < 1e-7
            else:
                assert rel_l2(o32.modules[j].g(s.name), ref) < 2e-5, s.name


# ------------------------------------------------------------------------------------------
# 2. library autograd transcription (unpadded, per sentence)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("adapters,split", [(True, True), (False, False)])
def test_against_autograd_transcription(adapters, split):
    setup = tiny_setup(adapters=adapters, split_enc=split)
    orc = tiny_oracle(setup)
    batch = tiny_batch(setup)
    for task in range(len(setup.tasks)):
        for m in orc.modules:
            m.grad[:] = 0
        loss = orc.train_step(task, batch.src_ids, batch.tgt_ids, batch.lengths)
        ref_loss, ref = torch_reference_step(orc, task, batch)
        assert abs(loss - ref_loss) < 1e-12 * abs(ref_loss)
        for (j, name), g in ref.items():
            got = orc.modules[j].g(name)
            assert np.abs(got - g).max() <= 1e-11 * max(1.0, np.abs(g).max()) + 1e-14, (j, name)


def test_adam_against_library_optimizer():
    setup = tiny_setup(adapters=False, split_enc=False)
    orc = tiny_oracle(setup)
    batch = tiny_batch(setup)
    ids = orc.routes[0]
    params = [torch.tensor(orc.modules[j].theta.copy(), requires_grad=True) for j in ids]
    opt = torch.optim.Adam(params, lr=3e-3, betas=(orc.b1, orc.b2), eps=orc.adam_eps)
    for step in range(3):
        orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
        for p, j in zip(params, ids):
            p.grad = torch.tensor(orc.modules[j].grad.copy())
        opt.step()
        orc.apply_update(None, 3e-3)
        for p, j in zip(params, ids):
            # the library folds the bias corrections in a different order: a few ulp
            np.testing.assert_allclose(orc.modules[j].theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)
            assert orc.modules[j].t == step + 1 and orc.modules[j].touched == 0
            assert not orc.modules[j].grad.any()


# ------------------------------------------------------------------------------------------
# 3. closed forms and brute force
# ------------------------------------------------------------------------------------------
def test_positional_table_values():
    pe = mo.positional_table(50, 16)
    for p, k in [(0, 0), (1, 0), (7, 3), (49, 7), (13, 5)]:
        ang = p / (10000.0 ** (2 * k / 16))
        assert pe[p, 2 * k] == pytest.approx(math.sin(ang), abs=1e-15)
        assert pe[p, 2 * k + 1] == pytest.approx(math.cos(ang), abs=1e-15)
    assert (pe[0, 0::2] == 0).all() and (pe[0, 1::2] == 1).all()


def test_layernorm_moments_and_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7, 32)) * 3 + 1
    y, _ = mo.layernorm_fwd(x, np.ones(32), np.zeros(32), 1e-6)
    assert np.abs(y.mean(-1)).max() < 1e-14
    var = x.var(-1)
    np.testing.assert_allclose((y * y).mean(-1), var / (var + 1e-6), rtol=1e-12)
    g, b = rng.standard_normal(32), rng.standard_normal(32)
    y, cache = mo.layernorm_fwd(x, g, b, 1e-6)
    ref = F.layer_norm(torch.tensor(x), (32,), torch.tensor(g), torch.tensor(b), 1e-6).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-13)
    dy = rng.standard_normal(x.shape)
    dx, dg, db = mo.layernorm_bwd(dy, cache, g)
    # per row: sum(dx) = 0, and sum(dx * xhat) = 0 when eps = 0 (then sum(xhat^2) = d exactly)
    assert np.abs(dx.sum(-1)).max() < 1e-12
    _, cache0 = mo.layernorm_fwd(x, g, b, 0.0)
    dx0, _, _ = mo.layernorm_bwd(dy, cache0, g)
    assert np.abs((dx0 * cache0[0]).sum(-1)).max() < 1e-12
    ref_dx, = torch.autograd.grad(
        F.layer_norm(xt := torch.tensor(x, requires_grad=True), (32,), torch.tensor(g), torch.tensor(b), 1e-6),
        xt, torch.tensor(dy))
    np.testing.assert_allclose(dx, ref_dx.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(db, dy.reshape(-1, 32).sum(0), rtol=1e-13)


def test_smoothed_ce_closed_forms_and_brute_force():
    rng = np.random.default_rng(1)
    U, V, eps = 6, 37, 0.1
    labels = rng.integers(0, V, U)
    # equal logits: loss = ln V whatever the label and eps
    rows, pq = mo.smoothed_ce(np.full((U, V), 0.3), labels, eps)
    np.testing.assert_allclose(rows, math.log(V), rtol=1e-14)
    z = rng.standard_normal((U, V)) * 2
    rows, pq = mo.smoothed_ce(z, labels, eps)
    assert np.abs(pq.sum(-1)).max() < 1e-14                       # sum_v dz = 0 per row
    for u in range(U):                                             # explicit -sum q log p
        logp = [z[u, v] - math.log(sum(math.exp(z[u, w]) for w in range(V))) for v in range(V)]
        q = [eps / V + (1 - eps if v == labels[u] else 0.0) for v in range(V)]
        assert rows[u] == pytest.approx(-sum(qv * lv for qv, lv in zip(q, logp)), rel=1e-13)
    ref = F.cross_entropy(torch.tensor(z), torch.tensor(labels), label_smoothing=eps, reduction="none")
    np.testing.assert_allclose(rows, ref.numpy(), rtol=1e-13)
    rows0, _ = mo.smoothed_ce(z, labels, 0.0)                      # eps = 0: plain NLL
    ref0 = F.nll_loss(F.log_softmax(torch.tensor(z), -1), torch.tensor(labels), reduction="none")
    np.testing.assert_allclose(rows0, ref0.numpy(), rtol=1e-13)


def test_initial_loss_is_log_vocab():
    """Zero generator => equal logits => loss ln V exactly; N(0,0.02) init => within 1e-2."""
    setup = tiny_setup(adapters=False, split_enc=False)
    orc = tiny_oracle(setup, perturbed=False)
    batch = tiny_batch(setup)
    assert abs(orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths) - math.log(setup.shape.vocab)) < 1e-2
    gen = orc.modules[orc.routes[0][4]]
    gen.theta[:] = 0
    assert orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths) == pytest.approx(math.log(setup.shape.vocab), rel=1e-14)


def test_single_key_attention_returns_value():
    rng = np.random.default_rng(2)
    d, H = 8, 2
    prm = [rng.standard_normal(s) for s in [(d, d), (d,)] * 4]
    xq, xkv = rng.standard_normal((1, 3, d)), rng.standard_normal((1, 1, d))
    y, cache = mo.attention_fwd(xq, xkv, prm, np.zeros((1, 3, 1), bool), H)
    v_row = xkv[0, 0] @ prm[4] + prm[5]
    np.testing.assert_allclose(y[0], np.tile(v_row @ prm[6] + prm[7], (3, 1)), rtol=1e-13)
    assert (cache[5] == 1.0).all()


def test_softmax_rows_masks_and_causality():
    setup = tiny_setup()
    orc = tiny_oracle(setup, keep_trace=True)
    batch = tiny_batch(setup)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    tr = orc.trace
    for P, blocked in ((tr["enc_P"], tr["enc_blocked"]), (tr["dec_self_P"], tr["dec_blocked"]),
                       (tr["dec_cross_P"], tr["cross_blocked"])):
        for p in P:
            assert np.abs(p.sum(-1) - 1).max() < 4e-16 * p.shape[-1]
            H = p.shape[1]
            assert (p[np.broadcast_to(blocked[:, None], p.shape)] == 0.0).all()   # exactly zero
    # the masks themselves, from their definition
    B = len(batch.lengths)
    for b in range(B):
        s_b, u_b = batch.lengths[b, 0], batch.lengths[b, 1] - 1
        for i in range(tr["dec_blocked"].shape[1]):
            for j in range(tr["dec_blocked"].shape[2]):
                assert tr["dec_blocked"][b, i, j] == (j > i or j >= u_b)
            for j in range(tr["cross_blocked"].shape[2]):
                assert tr["cross_blocked"][b, i, j] == (j >= s_b)
    # causality: changing target token p leaves per-token losses before p bit-identical
    base = tr["loss_rows"].copy()
    cu_u = mo.Oracle.packed_view(batch.src_ids, batch.tgt_ids, batch.lengths)["cu_u"]
    b, p = 1, 4
    tgt2 = batch.tgt_ids.copy()
    tgt2[b, p] = 3 + (tgt2[b, p] % 20)
    orc.train_step(0, batch.src_ids, tgt2, batch.lengths)
    new = orc.trace["loss_rows"]
    lo = cu_u[b]
    assert (new[lo:lo + p - 1] == base[lo:lo + p - 1]).all()       # labels before p, inputs before p
    assert new[lo + p - 1] != base[lo + p - 1]
    other = np.r_[0:lo, cu_u[b + 1]:len(base)]
    assert (new[other] == base[other]).all()


def test_adam_first_step_closed_form():
    """t=1: delta = -lr * g / (|g| + eps) ~ -lr*sign(g); exactly 0 where g = 0."""
    orc = mo.Oracle(16, 2, 32, 56, 12)
    j = orc.register_module("gen", init=np.arange(16 * 56 + 64, dtype=np.float64) * 1e-3)
    m = orc.modules[j]
    g = np.zeros(m.total)
    g[:10] = [1e-3, -2.0, 5e-7, -1e-9, 3.0, 0, 0, 1e-12, -1e-5, 7.0]
    m.grad[:] = g
    m.touched = 1
    before = m.theta.copy()
    orc.apply_update([j], 0.01)
    delta = m.theta - before
    np.testing.assert_allclose(delta, -0.01 * g / (np.abs(g) + 1e-9), rtol=1e-9, atol=1e-18)
    assert (delta[g == 0] == 0).all()
    assert m.t == 1


# ------------------------------------------------------------------------------------------
# 4. structural identities from the routing rules
# ------------------------------------------------------------------------------------------
def test_unused_modules_get_zero_gradient_and_no_update():
    """Alg. 1: a module outside the task's set has gradient 0; it takes no update."""
    setup = tiny_setup()
    orc = tiny_oracle(setup)
    batch = tiny_batch(setup)
    snap = [(m.theta.copy(), m.m.copy(), m.v.copy(), m.t) for m in orc.modules]
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    used = set(orc.routes[0])
    for j, m in enumerate(orc.modules):
        assert (m.touched == 1) == (j in used)
        if j not in used:
            assert not m.grad.any()
        else:
            assert m.grad.any()
    orc.apply_update(None, 1e-3)
    for j, (m, (th, mm, vv, t)) in enumerate(zip(orc.modules, snap)):
        if j in used:
            assert m.t == t + 1 and (m.theta != th).any()
        else:
            assert m.t == t and (m.theta == th).all() and (m.m == mm).all() and (m.v == vv).all()


def test_split_stack_equals_whole_stack():
    """h_i = T_i(h_{i-1}): two 1-layer modules in sequence == one 2-layer module."""
    split, whole = tiny_setup(adapters=False, split_enc=True), tiny_setup(adapters=False, split_enc=False)
    o_s, o_w = tiny_oracle(split), tiny_oracle(whole)
    batch = tiny_batch(split)
    r_s, r_w = o_s.routes[0], o_w.routes[0]
    e0, e1, ew = o_s.modules[r_s[1]], o_s.modules[r_s[2]], o_w.modules[r_w[1]]
    for s in ew.specs:                         # copy the whole stack's weights into the two halves
        if s.name.startswith("l0."):
            e0.p(s.name)[...] = ew.p(s.name)
        elif s.name.startswith("l1."):
            e1.p("l0." + s.name[3:])[...] = ew.p(s.name)
        else:
            e1.p(s.name)[...] = ew.p(s.name)
    for a, b in ((r_s[0], r_w[0]), (r_s[3], r_w[2]), (r_s[4], r_w[3]), (r_s[5], r_w[4])):
        o_s.modules[a].theta[:] = o_w.modules[b].theta
    l_s = o_s.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    l_w = o_w.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert l_s == l_w
    assert (e0.g("l0.self.Wq") == ew.g("l0.self.Wq")).all()
    assert (e1.g("l0.W2") == ew.g("l1.W2")).all()
    assert (e1.g("lnf.g") == ew.g("lnf.g")).all()
    assert (o_s.modules[r_s[0]].grad == o_w.modules[r_w[0]].grad).all()


def test_zero_adapter_is_identity():
    with_ad, without = tiny_setup(adapters=True), tiny_setup(adapters=False)
    o_a, o_n = tiny_oracle(with_ad), tiny_oracle(without)
    batch = tiny_batch(with_ad)
    ra, rn = o_a.routes[0], o_n.routes[0]
    for a, b in zip(ra[:6], rn):
        o_a.modules[a].theta[:] = o_n.modules[b].theta
    for a in ra[6:]:
        m = o_a.modules[a]
        for s in m.specs:
            if s.name.endswith(".Wu") or s.name.endswith(".bu"):
                m.p(s.name)[...] = 0
    la = o_a.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    ln_ = o_n.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    assert la == ln_
    for a, b in zip(ra[:6], rn):
        assert (o_a.modules[a].grad == o_n.modules[b].grad).all()


def test_padding_width_invariance_bit_exact():
    setup = tiny_setup()
    o1, o2 = tiny_oracle(setup), tiny_oracle(setup)
    batch = tiny_batch(setup, lengths=((5, 4), (3, 7), (6, 2)))
    src_w = np.pad(batch.src_ids, ((0, 0), (0, 3)))
    tgt_w = np.pad(batch.tgt_ids, ((0, 0), (0, 2)))
    l1 = o1.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    l2 = o2.train_step(0, src_w, tgt_w, batch.lengths)
    assert l1 == l2
    for a, b in zip(o1.modules, o2.modules):
        np.testing.assert_allclose(a.grad, b.grad, rtol=0, atol=1e-16)


def test_pad_rows_carry_zero_gradient():
    setup = tiny_setup()
    orc = tiny_oracle(setup, keep_trace=True)
    batch = tiny_batch(setup)
    orc.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    tr = orc.trace
    assert (tr["dx_src"][~tr["src_real"]] == 0).all()
    assert (tr["dy_tgt"][~tr["dec_real"]] == 0).all()
    assert not orc.modules[orc.routes[0][0]].g("E")[0].any()        # pad row of the table


def test_accumulation_counts_and_renormalisation():
    """Two identical steps then one update == one step then one update (g summed, / n_j)."""
    setup = tiny_setup()
    o1, o2 = tiny_oracle(setup), tiny_oracle(setup)
    batch = tiny_batch(setup)
    o1.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    for _ in range(2):
        o2.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    for j in o2.routes[0]:
        assert o2.modules[j].touched == 2
        if o2.modules[j].kind in ("src_emb", "tgt_emb"):   # row sums land one by one: rounding order
            np.testing.assert_allclose(o2.modules[j].grad, 2 * o1.modules[j].grad, rtol=1e-13, atol=1e-18)
        else:
            assert (o2.modules[j].grad == 2 * o1.modules[j].grad).all()
    o1.apply_update(None, 1e-3)
    o2.apply_update(None, 1e-3)
    for a, b in zip(o1.modules, o2.modules):
        assert a.t == b.t
        if a.kind in ("src_emb", "tgt_emb"):
            np.testing.assert_allclose(a.theta, b.theta, rtol=1e-12, atol=1e-12)
        else:
            assert (a.theta == b.theta).all()
    # two different tasks sharing modules: the shared encoder position is used twice
    o3 = tiny_oracle(tiny_setup(n_lang=3))
    t01 = 0                      # 0->1
    t21 = [n for n, _ in tiny_setup(n_lang=3).tasks].index("2-1")
    o3.train_step(t01, batch.src_ids, batch.tgt_ids, batch.lengths)
    o3.train_step(t21, batch.src_ids, batch.tgt_ids, batch.lengths)
    shared = set(o3.routes[t01]) & set(o3.routes[t21])
    assert shared and all(o3.modules[j].touched == 2 for j in shared)
    assert all(o3.modules[j].touched == 1 for j in set(o3.routes[t01]) ^ set(o3.routes[t21]))


def test_duplicated_batch_leaves_loss_unchanged():
    setup = tiny_setup()
    o1, o2 = tiny_oracle(setup), tiny_oracle(setup)
    batch = tiny_batch(setup)
    l1 = o1.train_step(0, batch.src_ids, batch.tgt_ids, batch.lengths)
    l2 = o2.train_step(0, np.tile(batch.src_ids, (2, 1)), np.tile(batch.tgt_ids, (2, 1)),
                       np.tile(batch.lengths, (2, 1)))
    assert l1 == pytest.approx(l2, rel=1e-14)
    assert rel_l2(o2.modules[o2.routes[0][1]].grad, o1.modules[o1.routes[0][1]].grad) < 1e-13


# ------------------------------------------------------------------------------------------
# 5. routes, layout, token bookkeeping
# ------------------------------------------------------------------------------------------
def test_route_rules():
    orc = mo.Oracle(16, 2, 32, 56, 12)
    se = orc.register_module("src_emb")
    x0 = orc.register_module("enc", "x", 0, 1, False)
    y1 = orc.register_module("enc", "y", 1, 1, True)
    y0 = orc.register_module("enc", "y", 0, 1, False)      # [x,y] and [y,x] need four modules
    x1 = orc.register_module("enc", "x", 1, 1, True)
    te = orc.register_module("tgt_emb")
    de = orc.register_module("dec", "t", 0, 2, True)
    ge = orc.register_module("gen")
    assert len({x0, y1, y0, x1}) == 4
    assert orc.route_task([se, x0, y1, te, de, ge]) == 0
    assert orc.route_task([se, y0, x1, te, de, ge]) == 1
    with pytest.raises(ValueError):       # a module at a position it was not defined for
        orc.route_task([se, y1, x0, te, de, ge])
    with pytest.raises(ValueError):       # different number of modules than the first task
        orc.route_task([se, x1, te, de, ge])
    with pytest.raises(ValueError):       # wrong order of kinds
        orc.route_task([x0, se, y1, te, de, ge])
    with pytest.raises(ValueError):       # stack not closed by its last position
        orc.route_task([se, x0, y0, te, de, ge])
    with pytest.raises(ValueError):
        orc.route_task([se, x0, y1, te, de, 99])
    assert orc.routes == [[se, x0, y1, te, de, ge], [se, y0, x1, te, de, ge]]


def test_layout_offsets_hand_computed():
    # d=64, F=256 encoder layer: every size is a multiple of 64, offsets are running sums
    specs, total = mo.module_layout("enc", 64, 256, 1000, n_layers=2, owns_final_norm=True)
    sizes = [64, 64] + [4096, 64] * 4 + [64, 64] + [64 * 256, 256, 256 * 64, 64]
    expect = np.concatenate([[0], np.cumsum(sizes * 2 + [64, 64])])
    assert [s.offset for s in specs] == expect[:-1].tolist() and total == expect[-1]
    assert specs[2].name == "l0.self.Wq" and specs[2].shape == (64, 64)
    assert specs[12].name == "l0.W1" and specs[12].shape == (64, 256)
    # generator with V=1000: Wg at 0 (64000), bg at 64000 (1000), total rounded up to 65024
    specs, total = mo.module_layout("gen", 64, 256, 1000)
    assert [(s.name, s.offset) for s in specs] == [("Wg", 0), ("bg", 64000)] and total == 65024
    # d=16: vectors of 16 still start on multiples of 64 elements
    specs, total = mo.module_layout("adapter", 16, 32, 56, n_layers=1, adapter_dim=8)
    assert [(s.name, s.offset) for s in specs] == [("l0.ln.g", 0), ("l0.ln.b", 64), ("l0.Wd", 128),
                                                   ("l0.bd", 256), ("l0.Wu", 320), ("l0.bu", 448)]
    assert total == 512
    dec, total = mo.module_layout("dec", 512, 2048, 32000, n_layers=6, owns_final_norm=True)
    per_layer = 3 * 1024 + 8 * (512 * 512 + 512) + 2 * 512 * 2048 + 2048 + 512
    assert total == 6 * per_layer + 1024 and len(dec) == 6 * 26 + 2


def test_packed_view_by_hand():
    src = np.array([[5, 6, 7], [8, 0, 0]], dtype=np.int32)
    tgt = np.array([[1, 9, 2, 0], [1, 4, 3, 2]], dtype=np.int32)
    lengths = np.array([[3, 3], [1, 4]], dtype=np.int32)
    pv = mo.Oracle.packed_view(src, tgt, lengths)
    assert pv["cu_s"].tolist() == [0, 3, 4] and pv["cu_u"].tolist() == [0, 2, 5]
    assert pv["src_tok"].tolist() == [5, 6, 7, 8] and pv["src_pos"].tolist() == [0, 1, 2, 0]
    assert pv["dec_tok"].tolist() == [1, 9, 1, 4, 3] and pv["label"].tolist() == [9, 2, 4, 3, 2]
    assert pv["dec_pos"].tolist() == [0, 1, 0, 1, 2]


def test_synthetic_inputs_shape_and_distribution():
    s2 = mm_synth.build_setup(2)
    batches = mm_synth.make_batches(s2, 4)
    for b in batches:
        B = len(b.lengths)
        assert B * b.lengths[:, 1].max() <= 4096 and b.n_tgt_tokens > 3000
        mo.Oracle.check_batch(b.src_ids, b.tgt_ids, b.lengths, 32000, 100)
        assert (b.tgt_ids[:, 0] == 1).all()
        assert all(b.tgt_ids[i, b.lengths[i, 1] - 1] == 2 for i in range(B))
        assert b.src_ids[b.src_ids > 0].min() >= 3
    ids = np.concatenate([b.src_ids[b.src_ids > 0] for b in batches])
    top = (ids == 3).mean()
    assert 0.10 < top < 0.18            # Zipf(1.1): the most frequent id carries ~14 % of tokens
    for idx, n_tasks in ((3, 12), (4, 8), (5, 56)):
        st = mm_synth.build_setup(idx)
        assert len(st.tasks) == n_tasks and len({tuple(t[1]) for t in st.tasks}) == n_tasks
        d = mm_synth.sample_directions(st, 50)
        assert d.min() >= 0 and d.max() < n_tasks
