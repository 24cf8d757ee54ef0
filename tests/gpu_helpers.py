"""Helpers for the GPU parity tests: build the GPU context and the CPU oracle from the same
seeded set-up, run the same batches through both, compare."""
from __future__ import annotations

import dataclasses
import sys

import numpy as np

import mm_synth
from oracle.mammoth_oracle import Oracle, build_from_setup


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def with_dtype(setup, dtype):
    return dataclasses.replace(setup, shape=dataclasses.replace(setup.shape, dtype=dtype))


def make_pair(setup, perturbed=True, keep_trace=False, max_batch_tokens=None):
    from paper_2403_07544_amd import context_from_setup
    ctx = context_from_setup(setup, fill_params=mm_synth.fill_params, perturbed=perturbed,
                             max_batch_tokens=max_batch_tokens)
    orc = build_from_setup(setup, dtype=np.float64, perturbed=perturbed, keep_trace=keep_trace,
                           fill_params=mm_synth.fill_params)
    return ctx, orc


def tensor_report(ctx, orc: Oracle, module_ids):
    """Per tensor: (module, name, rel_l2, cosine, ref_norm, abs_max_err, module_ref_norm)."""
    rows = []
    for j in module_ids:
        g = ctx.mm_get_grads(j).astype(np.float64)
        m = orc.modules[j]
        mod_norm = float(np.linalg.norm(m.grad))
        for s in m.specs:
            a = g[s.offset:s.offset + s.size]
            r = m.grad[s.offset:s.offset + s.size]
            nr, na = float(np.linalg.norm(r)), float(np.linalg.norm(a))
            err = float(np.linalg.norm(a - r))
            cos = float(a @ r / (na * nr)) if na > 0 and nr > 0 else 1.0 if na == nr else 0.0
            # the module's gradient norm scaled to this tensor's size: what the tensor's norm would be if
            # its elements had the module's root-mean-square size
            scale = mod_norm * (s.size / max(1, m.total)) ** 0.5
            rows.append((j, s.name, err / nr if nr > 0 else np.inf, cos, nr, float(np.abs(a - r).max()), scale, err, mod_norm))
        # alignment gaps must stay zero
        used = np.zeros(m.total, dtype=bool)
        for s in m.specs:
            used[s.offset:s.offset + s.size] = True
        assert not g[~used].any(), f"module {j}: gradient written into an alignment gap"
    return rows


def check_grads(ctx, orc, module_ids, rel_tol, cos_tol, floor_frac, label=""):
    """rel L2 <= rel_tol and cosine >= cos_tol per tensor.  A tensor whose elements are, by
    root-mean-square, below floor_frac of the size of its module's gradient elements (key biases:
    zero by the softmax's shift invariance) is instead required to have an error below rel_tol *
    floor_frac * (the module's gradient norm).  (The comparison is per element, so that a small vector such as a LayerNorm
    gain is not excused merely for being short next to a matrix.)"""
    worst = (0.0, None)
    under_floor = []
    for j, name, rel, cos, nr, amax, scale, err, mod_norm in tensor_report(ctx, orc, module_ids):
        if nr < floor_frac * scale:
            bound = rel_tol * floor_frac * mod_norm
            assert err <= bound, f"{label} module {j} {name}: error {err:.3e} vs bound {bound:.3e}"
            under_floor.append((name, nr / scale if scale > 0 else 0.0))
            continue
        assert rel <= rel_tol, f"{label} module {j} {name}: rel L2 {rel:.3e} > {rel_tol}"
        assert cos >= cos_tol, f"{label} module {j} {name}: cosine {cos:.6f} < {cos_tol}"
        if rel > worst[0]:
            worst = (rel, (j, name))
    if under_floor:
        kinds = sorted({n.split(".")[-1] for n, _ in under_floor})
        say(f"  {label}: {len(under_floor)} tensors whose elements are below {floor_frac:g} of their module's gradient elements (rms), checked by absolute error: "
            f"kinds {kinds}, largest share {max(f for _, f in under_floor):.2e}")
    return worst


def check_integer_artefacts(ctx, orc: Oracle, batch, task):
    """Routes, gather rows, labels, prefix sums and mask bitmaps: bit-exact."""
    pv = Oracle.packed_view(batch.src_ids, batch.tgt_ids, batch.lengths)
    assert ctx.mm_get_route(task) == orc.routes[task]
    for key_gpu, key_ref in (("cu_src", "cu_s"), ("cu_dec", "cu_u"), ("src_tok", "src_tok"),
                             ("src_pos", "src_pos"), ("dec_tok", "dec_tok"), ("dec_pos", "dec_pos"),
                             ("label", "label")):
        got = ctx.mm_debug_dump(key_gpu)
        assert got.dtype == np.int32 and np.array_equal(got, pv[key_ref].astype(np.int32)), key_gpu
    B, S_max = batch.src_ids.shape
    U_max = batch.tgt_ids.shape[1] - 1
    tr = orc.trace
    if tr:
        for key, blocked, shape in (("mask_enc", tr["enc_blocked"], (B, S_max, S_max)),
                                    ("mask_dec", tr["dec_blocked"], (B, U_max, U_max)),
                                    ("mask_cross", tr["cross_blocked"], (B, U_max, S_max))):
            got = ctx.mm_debug_dump(key).reshape(shape)
            assert np.array_equal(got.astype(bool), np.asarray(blocked)), key


def check_touched(ctx, orc):
    assert ctx.mm_get_touched().tolist() == [m.touched for m in orc.modules]


def check_untouched_zero(ctx, orc, used, never_used=None):
    """Modules off the route have an empty bucket; `never_used` (default: all of them, right for a
    context whose modules were not used and updated before) must not have had a byte of their
    bucket's memory written either."""
    for j in range(len(orc.modules)):
        if j not in used:
            assert not ctx.mm_get_grads(j).any(), f"module {j} is not on the route but has a gradient"
            if never_used is None or j in never_used:
                assert not ctx.mm_get_bucket_memory(j).any(), f"module {j} was never used but its bucket was written"
