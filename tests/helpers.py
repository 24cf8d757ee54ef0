"""Shared test helpers: tiny set-ups and an independent autograd transcription of the step.

The transcription (`torch_reference_step`) is a second opinion on the CPU oracle: it works on
unpadded sentences one at a time and takes LayerNorm, softmax, label-smoothed cross-entropy
and differentiation from the library, so it shares neither layout nor formulas with the
oracle's hand-written padded forward/backward.
"""
from __future__ import annotations

import math
from typing import Dict, Tuple

import numpy as np
import torch
import torch.nn.functional as F

import mm_synth
from mm_synth.configs import ModelShape, ModuleSpec, Setup
from oracle.mammoth_oracle import Oracle, build_from_setup


def tiny_setup(d=16, H=2, F_=32, V=56, n_lang=2, adapters=True, split_enc=True,
               enc_layers=(1, 1), dec_layers=2, max_len=12, seed=7, adapter_dim=8,
               dtype="f32") -> Setup:
    """Small model exercising every module kind: split encoder stack (language-specific
    position 0, shared position 1), language-specific decoders and optional adapters."""
    shape = ModelShape(d_model=d, n_heads=H, d_ff=F_, vocab=V, dtype=dtype, max_len=max_len,
                       batch_tokens=64)
    mods, ix = [], {}

    def add(key, spec):
        ix[key] = len(mods)
        mods.append(spec)

    for l in range(n_lang):
        add(("src_emb", l), ModuleSpec("src_emb", f"lang{l}"))
        if split_enc:
            add(("enc0", l), ModuleSpec("enc", f"lang{l}", 0, enc_layers[0], False))
        else:
            add(("enc0", l), ModuleSpec("enc", f"lang{l}", 0, sum(enc_layers), True))
        add(("tgt_emb", l), ModuleSpec("tgt_emb", f"lang{l}"))
        add(("dec", l), ModuleSpec("dec", f"lang{l}", 0, dec_layers, True))
        add(("gen", l), ModuleSpec("gen", f"lang{l}"))
        if adapters:
            add(("ad_enc", l), ModuleSpec("adapter", f"lang{l}", 0, sum(enc_layers), False, adapter_dim, "enc"))
            add(("ad_dec", l), ModuleSpec("adapter", f"lang{l}", 0, dec_layers, False, adapter_dim, "dec"))
    if split_enc:
        add(("enc1", 0), ModuleSpec("enc", "full", 1, enc_layers[1], True))
    tasks = []
    for s in range(n_lang):
        for t in range(n_lang):
            if s == t:
                continue
            ids = [ix[("src_emb", s)], ix[("enc0", s)]]
            if split_enc:
                ids.append(ix[("enc1", 0)])
            ids += [ix[("tgt_emb", t)], ix[("dec", t)], ix[("gen", t)]]
            if adapters:
                ids += [ix[("ad_enc", s)], ix[("ad_dec", t)]]
            tasks.append((f"{s}-{t}", ids))
    return Setup(0, "tiny test", shape, mods, tasks, 2, max_len, "uniform", fixed_batch=3,
                 pool_pairs=12, data_seed=seed, weight_seed=seed + 1, direction_seed=seed + 2)


def tiny_oracle(setup=None, dtype=np.float64, perturbed=True, keep_trace=False) -> Oracle:
    setup = setup or tiny_setup()
    return build_from_setup(setup, dtype=dtype, perturbed=perturbed, keep_trace=keep_trace,
                            fill_params=mm_synth.fill_params)


def tiny_batch(setup: Setup, lengths=((5, 4), (3, 7), (8, 2), (1, 5)), seed=3):
    return mm_synth.data.small_batch(setup.shape.vocab, lengths, seed)

def sharpen(orc: Oracle, scale: float, eos_shift: float):
    """Freshly initialised weights are so small that what the decoder writes hardly depends on
    the source.  Multiplying every matrix by `scale` makes the source, and the attention over
    it, decide the output; `eos_shift` is added to each generator's EOS bias to move where
    sentences stop.  (A test knob: trained weights are not available.)"""
    for m in orc.modules:
        if m.theta is None:
            continue
        for s in m.specs:
            if len(s.shape) == 2:
                m.p(s.name)[...] *= scale
        if m.kind == "gen":
            m.p("bg")[2] += eos_shift


# ----------------------------------------------------------------------------------------
def _pe(n, d):
    pos = torch.arange(n, dtype=torch.float64)[:, None]
    i2 = torch.arange(0, d, 2, dtype=torch.float64)[None, :]
    div = torch.exp(-math.log(10000.0) * i2 / d)
    pe = torch.zeros(n, d, dtype=torch.float64)
    pe[:, 0::2] = torch.sin(pos * div)
    pe[:, 1::2] = torch.cos(pos * div)
    return pe


def _mha(xq, xkv, W, pre, H, causal):
    d = xq.shape[-1]
    dh = d // H
    q = (xq @ W[pre + ".Wq"] + W[pre + ".bq"]).view(-1, H, dh).transpose(0, 1)
    k = (xkv @ W[pre + ".Wk"] + W[pre + ".bk"]).view(-1, H, dh).transpose(0, 1)
    v = (xkv @ W[pre + ".Wv"] + W[pre + ".bv"]).view(-1, H, dh).transpose(0, 1)
    s = q @ k.transpose(-1, -2) / math.sqrt(dh)
    if causal:
        n = s.shape[-1]
        s = s.masked_fill(~torch.tril(torch.ones(n, n, dtype=torch.bool)), float("-inf"))
    o = (F.softmax(s, dim=-1) @ v).transpose(0, 1).reshape(-1, d)
    return o @ W[pre + ".Wo"] + W[pre + ".bo"]


def _ffn(x, W, w1, b1, w2, b2):
    return F.relu(x @ W[w1] + W[b1]) @ W[w2] + W[b2]


def _sentence_logits(orc: Oracle, task: int, per_mod, src, dec_in):
    """Generator logits [len(dec_in), V] of one unpadded sentence pair, built from library
    layer_norm / softmax calls; `per_mod[j][name]` holds module j's tensors."""
    d, H, eps = orc.d, orc.H, orc.ln_eps
    i_src, enc_ids, i_tgt, dec_ids, i_gen, ad = orc.parse_route(orc.routes[task])

    def ln(x, W, name):
        return F.layer_norm(x, (d,), W[name + ".g"], W[name + ".b"], eps)

    def adapter(x, stack, li):
        if ad[stack] is None:
            return x
        W = per_mod[ad[stack]]
        return x + _ffn(ln(x, W, f"l{li}.ln"), W, f"l{li}.Wd", f"l{li}.bd", f"l{li}.Wu", f"l{li}.bu")

    x = math.sqrt(d) * per_mod[i_src]["E"][src] + _pe(len(src), d)
    li = 0
    for j in enc_ids:
        W = per_mod[j]
        for i in range(orc.modules[j].n_layers):
            a = ln(x, W, f"l{i}.ln1")
            x = x + _mha(a, a, W, f"l{i}.self", H, False)
            x = x + _ffn(ln(x, W, f"l{i}.ln2"), W, f"l{i}.W1", f"l{i}.b1", f"l{i}.W2", f"l{i}.b2")
            x = adapter(x, "enc", li)
            li += 1
    mem = ln(x, per_mod[enc_ids[-1]], "lnf")
    y = math.sqrt(d) * per_mod[i_tgt]["E"][dec_in] + _pe(len(dec_in), d)
    li = 0
    for j in dec_ids:
        W = per_mod[j]
        for i in range(orc.modules[j].n_layers):
            a = ln(y, W, f"l{i}.ln1")
            y = y + _mha(a, a, W, f"l{i}.self", H, True)
            y = y + _mha(ln(y, W, f"l{i}.ln2"), mem, W, f"l{i}.cross", H, False)
            y = y + _ffn(ln(y, W, f"l{i}.ln3"), W, f"l{i}.W1", f"l{i}.b1", f"l{i}.W2", f"l{i}.b2")
            y = adapter(y, "dec", li)
            li += 1
    h = ln(y, per_mod[dec_ids[-1]], "lnf")
    return h @ per_mod[i_gen]["Wg"] + per_mod[i_gen]["bg"]


def torch_reference_logits(orc: Oracle, task: int, src, dec_in) -> np.ndarray:
    """Logits of one unpadded sentence pair from the library transcription, as float64."""
    per_mod = {j: {s.name: torch.tensor(np.array(orc.modules[j].p(s.name), dtype=np.float64))
                   for s in orc.modules[j].specs} for j in orc.routes[task]}
    with torch.no_grad():
        z = _sentence_logits(orc, task, per_mod, torch.tensor(np.asarray(src, dtype=np.int64)),
                             torch.tensor(np.asarray(dec_in, dtype=np.int64)))
    return z.numpy()


def torch_reference_step(orc: Oracle, task: int, batch) -> Tuple[float, Dict[Tuple[int, str], np.ndarray]]:
    """Loss and gradient of every tensor of every module on the task's route."""
    d, H, eps = orc.d, orc.H, orc.ln_eps
    i_src, enc_ids, i_tgt, dec_ids, i_gen, ad = orc.parse_route(orc.routes[task])
    leaves: Dict[Tuple[int, str], torch.Tensor] = {}
    per_mod: Dict[int, Dict[str, torch.Tensor]] = {}
    for j in orc.routes[task]:
        per_mod[j] = {}
        for s in orc.modules[j].specs:
            t = torch.tensor(np.array(orc.modules[j].p(s.name), dtype=np.float64), requires_grad=True)
            leaves[(j, s.name)] = t
            per_mod[j][s.name] = t

    logits, labels = [], []
    for b in range(len(batch.lengths)):
        s_b, t_b = int(batch.lengths[b, 0]), int(batch.lengths[b, 1])
        src = torch.tensor(batch.src_ids[b, :s_b].astype(np.int64))
        tgt = torch.tensor(batch.tgt_ids[b, :t_b].astype(np.int64))
        logits.append(_sentence_logits(orc, task, per_mod, src, tgt[:-1]))
        labels.append(tgt[1:])
    loss = F.cross_entropy(torch.cat(logits), torch.cat(labels), label_smoothing=orc.eps_ls,
                           reduction="mean")
    loss.backward()
    grads = {k: (t.grad.numpy() if t.grad is not None else np.zeros(t.shape)) for k, t in leaves.items()}
    return float(loss.detach()), grads


def rel_l2(a, b):
    a, b = np.asarray(a, dtype=np.float64).ravel(), np.asarray(b, dtype=np.float64).ravel()
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a)
