"""Layerwise parameter-sharing patterns -> modules and task routes.

The paper (appendix B, "Layerwise parameter sharing") describes an architecture as two
concatenations of modules, one for the encoder and one for the decoder; each module position has
a number of layers and a sharing pattern, and the pattern fixes the *name* of the module a task
uses at that position: the constant "full", the cluster id of the source or target language, or
the source or target language code.  Tasks whose names agree at a position share that module.
Section 3.2 adds the two constraints the route table relies on: every task has the same number
of modules, and a module belongs to its sequential position (the groups [x, y] and [y, x] are
four modules, not two), which is what lets the layer counts be given per position
(`enc_layers`, `dec_layers`).

This file holds only that naming rule and the bookkeeping around it (host side, integers and
strings): embedding tables and generators are per language (source table by source language,
target table and generator by target language), as in every benchmark set-up here.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Sequence, Tuple

from .configs import ModuleSpec, Setup

PATTERNS = ("FULL", "SRC_GROUP", "TGT_GROUP", "GROUP", "SRC_LANGUAGE", "TGT_LANGUAGE", "LANGUAGE")


def sharing_name(pattern: str, stack: str, src: int, tgt: int, group_of: Dict[int, int]) -> str:
    """Name of the module a task (src -> tgt) uses at a position with this pattern.

    GROUP and LANGUAGE are the conveniences of appendix B: the source-side variant in the
    encoder, the target-side variant in the decoder.  A target-side pattern in the encoder (or a
    source-side one in the decoder) is allowed, as the appendix notes.
    """
    if pattern not in PATTERNS:
        raise ValueError(f"unknown sharing pattern {pattern!r}")
    if stack not in ("enc", "dec"):
        raise ValueError(f"stack must be 'enc' or 'dec', not {stack!r}")
    if pattern == "GROUP":
        pattern = "SRC_GROUP" if stack == "enc" else "TGT_GROUP"
    if pattern == "LANGUAGE":
        pattern = "SRC_LANGUAGE" if stack == "enc" else "TGT_LANGUAGE"
    if pattern == "FULL":
        return "full"
    lang = src if pattern.startswith("SRC") else tgt
    if pattern.endswith("GROUP"):
        if lang not in group_of:
            raise ValueError(f"language {lang} has no group")
        return f"group{group_of[lang]}"
    return f"lang{lang}"


def layerwise_tasks(pairs: Sequence[Tuple[int, int]], enc: Sequence[Tuple[str, int]],
                    dec: Sequence[Tuple[str, int]], group_of: Dict[int, int] | None = None):
    """Modules and routes of the tasks `pairs` under a layerwise sharing definition.

    enc / dec: one (pattern, n_layers) per module position, in order (`enc_layers` /
    `dec_layers` are the second members).  Returns (modules, tasks): `modules` in order of first
    use, `tasks` as (name, ordered module indices: source table, encoder positions, target table,
    decoder positions, generator) -- the order `mm_route_task` takes.  The last position of a
    stack carries the stack's closing LayerNorm.  Every task gets len(enc) + len(dec) + 3
    modules, so the same-count constraint holds by construction.
    """
    if not enc or not dec:
        raise ValueError("each stack needs at least one module position")
    for pattern, n_layers in list(enc) + list(dec):
        if pattern not in PATTERNS:
            raise ValueError(f"unknown sharing pattern {pattern!r}")
        if n_layers < 1:
            raise ValueError("a module position has at least one layer")
    group_of = group_of or {}
    modules: List[ModuleSpec] = []
    index: Dict[Tuple[str, int, str], int] = {}   # (kind, position, name): position-specific

    def module(kind: str, position: int, name: str, n_layers: int = 0, last: bool = False) -> int:
        key = (kind, position, name)
        if key not in index:
            index[key] = len(modules)
            modules.append(ModuleSpec(kind=kind, name=name, position=position, n_layers=n_layers,
                                      owns_final_norm=last))
        return index[key]

    tasks = []
    for s, t in pairs:
        route = [module("src_emb", 0, f"lang{s}")]
        for pos, (pattern, n_layers) in enumerate(enc):
            route.append(module("enc", pos, sharing_name(pattern, "enc", s, t, group_of), n_layers,
                                pos == len(enc) - 1))
        route.append(module("tgt_emb", 0, f"lang{t}"))
        for pos, (pattern, n_layers) in enumerate(dec):
            route.append(module("dec", pos, sharing_name(pattern, "dec", s, t, group_of), n_layers,
                                pos == len(dec) - 1))
        route.append(module("gen", 0, f"lang{t}"))
        tasks.append((f"{s}-{t}", route))
    return modules, tasks


def route_signature(modules: Sequence[ModuleSpec], route: Sequence[int]):
    """What a route means, independent of how the module list happens to be numbered."""
    return [(modules[j].kind, modules[j].position, modules[j].name, modules[j].n_layers,
             modules[j].owns_final_norm) for j in route]


def parse_stack(text: str) -> List[Tuple[str, int]]:
    """"LANGUAGE:4,FULL:4" -> [("LANGUAGE", 4), ("FULL", 4)] (pattern:layers per module position)."""
    out = []
    for item in text.split(","):
        pattern, _, layers = item.strip().partition(":")
        if pattern not in PATTERNS or not layers.isdigit() or int(layers) < 1:
            raise ValueError(f"expected PATTERN:LAYERS with PATTERN one of {', '.join(PATTERNS)}; got {item!r}")
        out.append((pattern, int(layers)))
    return out


def pattern_setup(base: Setup, n_lang: int, enc: Sequence[Tuple[str, int]], dec: Sequence[Tuple[str, int]],
                  group_of: Dict[int, int] | None = None) -> Setup:
    """A set-up with `base`'s model shape, data recipe and seeds, and the modules and tasks (all
    ordered pairs of `n_lang` languages) that the layerwise sharing definition gives."""
    if n_lang < 2:
        raise ValueError("a translation direction needs two languages")
    pairs = [(s, t) for s in range(n_lang) for t in range(n_lang) if s != t]
    modules, tasks = layerwise_tasks(pairs, enc, dec, group_of)
    title = "enc " + ",".join(f"{p}:{n}" for p, n in enc) + " / dec " + ",".join(f"{p}:{n}" for p, n in dec)
    return dataclasses.replace(base, title=f"{n_lang} languages, {title}", modules=modules, tasks=tasks)
