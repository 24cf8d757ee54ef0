"""The five benchmark set-ups: model shape, resident modules and tasks (directions).

A *task* is one translation direction; it names, in order, the modules its batches run
through (paper section 3.2, "Design principles": a task fixes a set of modules; module
definitions are specific to a sequential position; every task has the same number of
modules; the number of layers is a property of the module position).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    dtype: str  # "f32" or "bf16" (storage of activations / working weights on the GPU)
    max_len: int
    batch_tokens: int  # budget on B * max target length of a batch
    label_smoothing: float = 0.1
    adam_beta1: float = 0.9
    adam_beta2: float = 0.98
    adam_eps: float = 1e-9
    ln_eps: float = 1e-6
    lr: float = 2e-4


@dataclass(frozen=True)
class ModuleSpec:
    kind: str  # "src_emb" | "enc" | "tgt_emb" | "dec" | "gen" | "adapter"
    name: str  # sharing-group name, e.g. "lang2", "group0", "full"
    position: int = 0  # index in the encoder / decoder module sequence
    n_layers: int = 0  # layers of this module (enc/dec), layers covered (adapter)
    owns_final_norm: bool = False  # last position of a stack carries the closing LayerNorm
    adapter_dim: int = 0
    stack: str = ""  # adapters only: "enc" or "dec"


@dataclass
class Setup:
    index: int
    title: str
    shape: ModelShape
    modules: List[ModuleSpec]
    # task = (name, ordered module indices: src_emb, enc[0..], tgt_emb, dec[0..], gen, adapters...)
    tasks: List[Tuple[str, List[int]]]
    len_lo: int
    len_hi: int
    len_mode: str  # "uniform" (independent src/tgt) or "loguniform" (correlated)
    fixed_batch: int = 0  # >0: batches of exactly this many pairs, no length bucketing
    pool_pairs: int = 16384
    data_seed: int = 0
    weight_seed: int = 0
    direction_seed: int = 0
    extra: dict = field(default_factory=dict)


_BASE = dict(d_model=512, n_heads=8, d_ff=2048, vocab=32000, dtype="bf16", max_len=100,
             batch_tokens=4096)


def _seeds(index: int) -> dict:
    base = 0x4D4D0000 + index
    return dict(data_seed=base, weight_seed=base + 0x100, direction_seed=base + 0x200)


def _lang_specific(n_lang: int, n_layers: int):
    """src_emb, enc, tgt_emb, dec, gen per language; returns (modules, lookup)."""
    mods: List[ModuleSpec] = []
    ix = {}
    for l in range(n_lang):
        for kind in ("src_emb", "enc", "tgt_emb", "dec", "gen"):
            ix[(kind, l)] = len(mods)
            mods.append(ModuleSpec(kind=kind, name=f"lang{l}", position=0,
                                   n_layers=n_layers if kind in ("enc", "dec") else 0,
                                   owns_final_norm=kind in ("enc", "dec")))
    return mods, ix


def _pairs(n_lang: int):
    return [(s, t) for s in range(n_lang) for t in range(n_lang) if s != t]


def build_setup(index: int) -> Setup:
    """index 1..5 as in the benchmark definition."""
    if index == 1:
        shape = ModelShape(d_model=64, n_heads=4, d_ff=256, vocab=1000, dtype="f32", max_len=20,
                           batch_tokens=8 * 20)
        mods = [ModuleSpec("src_emb", "lang0"), ModuleSpec("enc", "lang0", 0, 2, True),
                ModuleSpec("tgt_emb", "lang1"), ModuleSpec("dec", "lang1", 0, 2, True),
                ModuleSpec("gen", "lang1")]
        return Setup(1, "tiny fp32 single task", shape, mods, [("0-1", [0, 1, 2, 3, 4])],
                     5, 20, "uniform", fixed_batch=8, pool_pairs=8 * 32, **_seeds(1))
    if index == 2:
        shape = ModelShape(**_BASE)
        mods = [ModuleSpec("src_emb", "lang0"), ModuleSpec("enc", "lang0", 0, 6, True),
                ModuleSpec("tgt_emb", "lang1"), ModuleSpec("dec", "lang1", 0, 6, True),
                ModuleSpec("gen", "lang1")]
        return Setup(2, "Transformer-base single task bf16", shape, mods,
                     [("0-1", [0, 1, 2, 3, 4])], 10, 100, "loguniform", **_seeds(2))
    if index == 3:
        shape = ModelShape(**_BASE)
        mods, ix = _lang_specific(4, 6)
        tasks = [(f"{s}-{t}", [ix[("src_emb", s)], ix[("enc", s)], ix[("tgt_emb", t)],
                               ix[("dec", t)], ix[("gen", t)]]) for s, t in _pairs(4)]
        return Setup(3, "fully modular bf16", shape, mods, tasks, 10, 100, "loguniform",
                     **_seeds(3))
    if index == 4:
        shape = ModelShape(**_BASE)
        group_of = {0: 0, 1: 0, 2: 1, 3: 1}
        mods: List[ModuleSpec] = []
        ix = {}

        def add(key, spec):
            ix[key] = len(mods)
            mods.append(spec)

        for l in range(4):
            add(("src_emb", l), ModuleSpec("src_emb", f"lang{l}"))
        for g in range(2):
            add(("enc0", g), ModuleSpec("enc", f"group{g}", 0, 3, False))
        add(("enc1", 0), ModuleSpec("enc", "full", 1, 3, True))
        for l in range(4):
            add(("tgt_emb", l), ModuleSpec("tgt_emb", f"lang{l}"))
            add(("dec", l), ModuleSpec("dec", f"lang{l}", 0, 6, True))
            add(("gen", l), ModuleSpec("gen", f"lang{l}"))
        for l in range(4):
            add(("ad_enc", l), ModuleSpec("adapter", f"lang{l}", 0, 6, False, 64, "enc"))
            add(("ad_dec", l), ModuleSpec("adapter", f"lang{l}", 0, 6, False, 64, "dec"))
        seeds = _seeds(4)
        order = np.random.Generator(np.random.Philox(key=seeds["direction_seed"])).permutation(12)
        pairs = [_pairs(4)[i] for i in order[:8]]
        tasks = [(f"{s}-{t}", [ix[("src_emb", s)], ix[("enc0", group_of[s])], ix[("enc1", 0)],
                               ix[("tgt_emb", t)], ix[("dec", t)], ix[("gen", t)],
                               ix[("ad_enc", s)], ix[("ad_dec", t)]]) for s, t in pairs]
        return Setup(4, "partially shared bf16 with adapters", shape, mods, tasks, 10, 100,
                     "loguniform", **seeds)
    if index == 5:
        shape = ModelShape(d_model=1024, n_heads=16, d_ff=4096, vocab=64000, dtype="bf16",
                           max_len=200, batch_tokens=8192)
        mods, ix = _lang_specific(8, 6)
        tasks = [(f"{s}-{t}", [ix[("src_emb", s)], ix[("enc", s)], ix[("tgt_emb", t)],
                               ix[("dec", t)], ix[("gen", t)]]) for s, t in _pairs(8)]
        return Setup(5, "Transformer-big bf16, one GPU's share", shape, mods, tasks, 10, 200,
                     "loguniform", **_seeds(5))
    if index in (6, 7, 8):
        # The paper's own benchmark shapes (section 4): d=512, 8 heads, FFN 2048, 64k vocabulary,
        # maximum length 200, 4096-token batches; four languages resident as one GPU's share.
        shape = ModelShape(d_model=512, n_heads=8, d_ff=2048, vocab=64000, dtype="bf16", max_len=200,
                           batch_tokens=4096)
        n_lang = 4
        mods: List[ModuleSpec] = []
        ix = {}

        def add(key, spec):
            ix[key] = len(mods)
            mods.append(spec)

        enc_split = {6: None, 7: (4, 4), 8: None}[index]
        enc_layers = {6: 6, 7: 8, 8: 9}[index]
        dec_layers = {6: 6, 7: 4, 8: 4}[index]
        for l in range(n_lang):
            add(("src_emb", l), ModuleSpec("src_emb", f"lang{l}"))
            add(("tgt_emb", l), ModuleSpec("tgt_emb", f"lang{l}"))
            add(("dec", l), ModuleSpec("dec", f"lang{l}", 0, dec_layers, True))
            add(("gen", l), ModuleSpec("gen", f"lang{l}"))
            if index == 6:
                add(("enc0", l), ModuleSpec("enc", f"lang{l}", 0, enc_layers, True))
            elif index == 7:
                add(("enc0", l), ModuleSpec("enc", f"lang{l}", 0, enc_split[0], False))
        if index == 7:
            add(("enc1", 0), ModuleSpec("enc", "full", 1, enc_split[1], True))
        if index == 8:
            add(("enc0", 0), ModuleSpec("enc", "full", 0, enc_layers, True))
        tasks = []
        for s_, t_ in _pairs(n_lang):
            enc = [ix[("enc0", s_ if index != 8 else 0)]] + ([ix[("enc1", 0)]] if index == 7 else [])
            tasks.append((f"{s_}-{t_}", [ix[("src_emb", s_)]] + enc + [ix[("tgt_emb", t_)], ix[("dec", t_)], ix[("gen", t_)]]))
        title = {6: "paper shape: language-specific 6+6, 64k vocab", 7: "paper shape: 4 language-specific + 4 shared encoder layers, 4 decoder layers",
                 8: "paper shape: shared 9-layer encoder, 4-layer language-specific decoders"}[index]
        return Setup(index, title, shape, mods, tasks, 10, 200, "loguniform", **_seeds(index))
    raise ValueError(f"no such setup: {index}")


CONFIGS = (1, 2, 3, 4, 5)
PAPER_SHAPES = (6, 7, 8)
