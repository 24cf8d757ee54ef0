"""Host-side logic of the library, exercised without a GPU through plan-only contexts: exported
symbols, bucket layouts, route rules (paper section 3.2), batch validation, error codes."""
import ctypes
import re
import os

import numpy as np
import pytest

import mm_synth
from oracle.mammoth_oracle import Oracle, module_layout
from paper_2403_07544_amd import (Context, MMError, context_from_setup, load_library, EXPORTS, MM_EINVAL,
                                  MM_ERANGE, MM_ESTATE)
from tests.helpers import tiny_batch, tiny_setup

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mammoth_hip.h")).read()
    declared = set(re.findall(r"\b(mm_[a-z_]+)\s*\(", header))
    assert declared == set(EXPORTS)
    lib = load_library()
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_bucket_layout_matches_oracle_bit_exactly(index):
    setup = mm_synth.build_setup(index)
    ctx = context_from_setup(setup, plan_only=True)
    sh = setup.shape
    for j, ms in enumerate(setup.modules):
        specs, total = module_layout(ms.kind, sh.d_model, sh.d_ff, sh.vocab, ms.n_layers, ms.owns_final_norm,
                                     ms.adapter_dim)
        table, got_total = ctx.mm_get_layout(j)
        assert got_total == total
        assert [(r, o, rows * cols) for r, o, rows, cols in table] == [(s.role, s.offset, s.size) for s in specs]
        for (r, o, rows, cols), s in zip(table, specs):
            assert (rows, cols) == (s.shape if len(s.shape) == 2 else (1, s.shape[0]))
    for t, (_, ids) in enumerate(setup.tasks):
        assert ctx.mm_get_route(t) == ids
    assert ctx.mm_get_touched().tolist() == [0] * len(setup.modules)


def _ctx():
    return Context(32, 2, 64, 56, "f32", max_len=24, max_batch_tokens=256, plan_only=True)


def test_route_rules_match_oracle():
    ctx = _ctx()
    orc = Oracle(32, 2, 64, 56, 24)
    mods = [("src_emb", "s", 0, 0, False), ("enc", "x", 0, 1, False), ("enc", "y", 1, 1, True),
            ("enc", "y", 0, 1, False), ("enc", "x", 1, 1, True), ("tgt_emb", "t", 0, 0, False),
            ("dec", "t", 0, 2, True), ("gen", "t", 0, 0, False), ("enc", "whole", 0, 2, True)]
    for kind, name, pos, nl, fin in mods:
        a = ctx.mm_register_module(kind, name, pos, nl, fin)
        b = orc.register_module(kind, name, pos, nl, fin)
        assert a == b
    ad_ok = ctx.mm_register_module("adapter", "a", 0, 2, False, 16, "enc")
    ad_short = ctx.mm_register_module("adapter", "a", 0, 1, False, 16, "enc")
    orc.register_module("adapter", "a", 0, 2, False, 16, "enc")
    orc.register_module("adapter", "a", 0, 1, False, 16, "enc")
    good = [[0, 1, 2, 5, 6, 7, ad_ok], [0, 3, 4, 5, 6, 7, ad_ok]]
    bad = [[0, 2, 1, 5, 6, 7, ad_ok],      # positions swapped
           [0, 1, 2, 5, 6, 7],             # fewer modules than the first task
           [1, 0, 2, 5, 6, 7, ad_ok],      # kinds out of order
           [0, 1, 3, 5, 6, 7, ad_ok],      # stack not closed by its last position
           [0, 1, 2, 5, 6, 99, ad_ok],     # unknown id
           [0, 1, 2, 5, 6, 7, ad_short],   # adapter does not cover the stack
           [0, 1, 2, 5, 6, 7, 7]]          # duplicate
    for ids in good:
        assert ctx.mm_route_task(ids) == orc.route_task(ids)
    for ids in bad:
        with pytest.raises(MMError) as ei:
            ctx.mm_route_task(ids)
        assert ei.value.status == MM_EINVAL
        with pytest.raises(ValueError):
            orc.route_task(ids)
    assert ctx.mm_get_route(0) == good[0] and ctx.mm_get_route(1) == good[1]
    with pytest.raises(MMError):
        ctx.mm_get_route(2)


def test_batch_validation_and_state_errors():
    setup = tiny_setup(d=32, H=2, F_=64, V=56, adapter_dim=16, max_len=24)
    ctx = context_from_setup(setup, plan_only=True, max_batch_tokens=64)
    batch = tiny_batch(setup)

    def status(**kw):
        args = dict(task=0, src=batch.src_ids, tgt=batch.tgt_ids, lengths=batch.lengths)
        args.update(kw)
        with pytest.raises(MMError) as ei:
            ctx.mm_train_step(args["task"], args["src"], args["tgt"], args["lengths"])
        return ei.value.status

    assert status() == MM_ESTATE                       # valid batch, but the context cannot compute
    assert status(task=7) == MM_EINVAL
    assert status(src=batch.src_ids[:0], tgt=batch.tgt_ids[:0], lengths=batch.lengths[:0]) == MM_EINVAL   # empty batch
    src = batch.src_ids.copy(); src[0, 0] = 56
    assert status(src=src) == MM_ERANGE                # id >= vocab
    tgt = batch.tgt_ids.copy(); tgt[0, -1] = 5
    assert status(tgt=tgt) == MM_ERANGE                # non-pad after the end
    ln = batch.lengths.copy(); ln[1, 0] = 0
    assert status(lengths=ln) == MM_ERANGE
    ln = batch.lengths.copy(); ln[1, 1] = 1
    assert status(lengths=ln) == MM_ERANGE
    wide = np.pad(batch.src_ids, ((0, 0), (0, 30)))
    assert status(src=wide) == MM_ERANGE               # wider than max_len
    big = mm_synth.data.small_batch(56, [(20, 20)] * 4, 1)
    assert status(src=big.src_ids, tgt=big.tgt_ids, lengths=big.lengths) == MM_ERANGE  # > max_batch_tokens
    with pytest.raises(MMError) as ei:
        ctx.mm_apply_update(None, 1e-3)
    assert ei.value.status == MM_ESTATE
    with pytest.raises(MMError) as ei:
        ctx.mm_get_params(0)
    assert ei.value.status == MM_ESTATE


def test_create_rejects_bad_shapes():
    for kw in (dict(d_model=30), dict(n_heads=3), dict(vocab=57), dict(max_len=300), dict(max_batch_tokens=20000),
               dict(d_ff=50)):
        args = dict(d_model=32, n_heads=2, d_ff=64, vocab=56, dtype="f32", max_len=24, max_batch_tokens=256,
                    plan_only=True)
        args.update(kw)
        with pytest.raises(MMError) as ei:
            Context(**args)
        assert ei.value.status == MM_EINVAL
    ctx = _ctx()
    with pytest.raises(MMError):
        ctx.mm_register_module("adapter", "a", 0, 2, False, 10, "enc")   # bottleneck not a multiple of 16
    with pytest.raises(MMError):
        ctx.mm_register_module("enc", "e", 0, 0, True)                   # no layers
    j = ctx.mm_register_module("gen", "g")
    with pytest.raises(MMError):
        ctx.mm_register_module("gen", "g", init=np.zeros(10, dtype=np.float32))  # wrong length
    assert ctx.mm_get_layout(j)[1] == 32 * 56 + 64


def test_temperature_task_sampling():
    """Skewed-data sampling of the bench: probabilities follow size^(1/T) with sizes ~ 1/rank."""
    p1 = mm_synth.task_probabilities(4, 1.0)
    assert np.allclose(p1, np.array([1, 1 / 2, 1 / 3, 1 / 4]) / (25 / 12))
    p2 = mm_synth.task_probabilities(4, 2.0)
    assert np.allclose(p2 / p2[0], np.array([1, 2 ** -0.5, 3 ** -0.5, 0.5]))
    assert np.allclose(mm_synth.task_probabilities(7, 1e9), 1 / 7, atol=1e-6)
    st = mm_synth.build_setup(3)
    d = mm_synth.sample_directions(st, 20000, temperature=1.0)
    assert d.min() >= 0 and d.max() < len(st.tasks)
    freq = np.bincount(d, minlength=len(st.tasks)) / len(d)
    assert np.abs(freq - mm_synth.task_probabilities(len(st.tasks), 1.0)).max() < 0.01
    assert np.array_equal(d, mm_synth.sample_directions(st, 20000, temperature=1.0))     # seeded
    assert np.array_equal(mm_synth.sample_directions(st, 50), mm_synth.sample_directions(st, 50))


def test_paper_shape_setups_carry_section4_numbers():
    """Set-ups 6-8 against the figures section 4 of the paper prints (tests/golden)."""
    gold = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_section4_shapes.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            gold[k.strip()] = int(v)
    for index, scheme in ((6, 1), (7, 2), (8, 3)):
        st = mm_synth.build_setup(index)
        sh = st.shape
        assert (sh.vocab, sh.d_model, sh.n_heads, sh.d_ff, sh.max_len, sh.batch_tokens) == tuple(
            gold[k] for k in ("vocab", "d_model", "n_heads", "d_ff", "max_len", "batch_tokens"))
        for name, ids in st.tasks:
            enc = [st.modules[j] for j in ids if st.modules[j].kind == "enc"]
            dec = [st.modules[j] for j in ids if st.modules[j].kind == "dec"]
            assert sum(m.n_layers for m in enc) == gold[f"scheme{scheme}_enc_layers"], name
            assert sum(m.n_layers for m in dec) == gold[f"scheme{scheme}_dec_layers"], name
        names = {m.name for m in st.modules if m.kind == "enc"}
        if scheme == 1:      # one encoder per language, none shared
            assert "full" not in names and len(names) == 4
        if scheme == 2:      # a language-specific first half, a second half shared by all
            shared = [m for m in st.modules if m.kind == "enc" and m.name == "full"]
            assert len(shared) == 1 and shared[0].n_layers == gold["scheme2_enc_shared"] and shared[0].position == 1
        if scheme == 3:      # one encoder for all languages
            assert names == {"full"}


# ---- layerwise sharing patterns (appendix B) and the task constraints of section 3.2 ----------

def _all_pairs(n):
    return [(s, t) for s in range(n) for t in range(n) if s != t]


# (set-up, encoder positions, decoder positions, language groups): the sharing definition each
# benchmark set-up is meant to be an instance of
_SHARING = {
    3: ([("LANGUAGE", 6)], [("LANGUAGE", 6)], None),
    4: ([("GROUP", 3), ("FULL", 3)], [("LANGUAGE", 6)], {0: 0, 1: 0, 2: 1, 3: 1}),
    5: ([("SRC_LANGUAGE", 6)], [("TGT_LANGUAGE", 6)], None),
    6: ([("LANGUAGE", 6)], [("LANGUAGE", 6)], None),
    7: ([("LANGUAGE", 4), ("FULL", 4)], [("LANGUAGE", 4)], None),
    8: ([("FULL", 9)], [("LANGUAGE", 4)], None),
}


@pytest.mark.parametrize("index", sorted(_SHARING))
def test_benchmark_routes_are_instances_of_the_sharing_patterns(index):
    setup = mm_synth.build_setup(index)
    enc, dec, groups = _SHARING[index]
    pairs = [tuple(int(x) for x in name.split("-")) for name, _ in setup.tasks]
    modules, tasks = mm_synth.layerwise_tasks(pairs, enc, dec, groups)
    n_route = len(enc) + len(dec) + 3
    for (name, route), (name2, route2) in zip(setup.tasks, tasks):
        assert name == name2
        # adapters (set-up 4) follow the pattern-defined part of a route
        assert mm_synth.route_signature(setup.modules, route[:n_route]) == mm_synth.route_signature(modules, route2)
        assert all(setup.modules[j].kind == "adapter" for j in route[n_route:])
    # the same modules exist, whatever their numbering (a set-up may hold modules no task uses yet)
    have = {mm_synth.route_signature(setup.modules, [j])[0] for j, m in enumerate(setup.modules) if m.kind != "adapter"}
    used = {mm_synth.route_signature(modules, [j])[0] for j in range(len(modules))}
    assert used <= have
    if index != 4:   # set-up 4 keeps all four languages resident but trains 8 of the 12 directions
        assert used == have


def test_sharing_pattern_names():
    g = {0: 0, 1: 0, 2: 1}
    name = mm_synth.sharing_name
    assert name("FULL", "enc", 0, 2, g) == name("FULL", "dec", 1, 0, g) == "full"
    assert name("SRC_GROUP", "enc", 1, 2, g) == "group0" and name("TGT_GROUP", "enc", 1, 2, g) == "group1"
    assert name("GROUP", "enc", 1, 2, g) == "group0" and name("GROUP", "dec", 1, 2, g) == "group1"
    assert name("SRC_LANGUAGE", "dec", 1, 2, g) == "lang1" and name("TGT_LANGUAGE", "enc", 1, 2, g) == "lang2"
    assert name("LANGUAGE", "enc", 1, 2, g) == "lang1" and name("LANGUAGE", "dec", 1, 2, g) == "lang2"
    with pytest.raises(ValueError):
        name("HALF", "enc", 0, 1, g)
    with pytest.raises(ValueError):
        name("SRC_GROUP", "enc", 5, 1, g)   # a language outside every cluster


def test_modules_are_position_specific_and_counts_are_equal():
    # two positions with the same pattern: the names coincide, the modules do not (section 3.2:
    # the groups [x, y] and [y, x] are four modules)
    modules, tasks = mm_synth.layerwise_tasks([(0, 1), (1, 0)], [("SRC_LANGUAGE", 2), ("TGT_LANGUAGE", 2)],
                                              [("FULL", 1)], None)
    enc = [m for m in modules if m.kind == "enc"]
    assert sorted((m.position, m.name) for m in enc) == [(0, "lang0"), (0, "lang1"), (1, "lang0"), (1, "lang1")]
    assert len({len(r) for _, r in tasks}) == 1                       # constraint (i)
    assert [m.owns_final_norm for m in enc] == [m.position == 1 for m in enc]
    assert sum(m.kind == "dec" for m in modules) == 1                 # one fully shared decoder
    # a target-language-dependent encoder position: tasks into the same language share it
    modules, tasks = mm_synth.layerwise_tasks(_all_pairs(3), [("LANGUAGE", 1), ("TGT_LANGUAGE", 1)], [("FULL", 1)])
    by_name = dict(tasks)
    assert by_name["0-2"][2] == by_name["1-2"][2] != by_name["0-1"][2]
    assert by_name["0-2"][1] == by_name["0-1"][1] != by_name["1-2"][1]


def test_pattern_generated_tasks_register_and_route():
    # what the helper emits passes the library's own route rules (same count for every task, kinds
    # in order, positions consistent, stacks closed) -- host bookkeeping only, no compute
    modules, tasks = mm_synth.layerwise_tasks(_all_pairs(3), [("GROUP", 1), ("FULL", 1)], [("LANGUAGE", 2)],
                                              {0: 0, 1: 0, 2: 1})
    ctx = _ctx()
    orc = Oracle(32, 2, 64, 56, 24)
    for m in modules:
        a = ctx.mm_register_module(m.kind, m.name, m.position, m.n_layers, m.owns_final_norm)
        assert a == orc.register_module(m.kind, m.name, m.position, m.n_layers, m.owns_final_norm)
    for k, (_, route) in enumerate(tasks):
        assert ctx.mm_route_task(route) == orc.route_task(route) == k
        assert ctx.mm_get_route(k) == list(route)
