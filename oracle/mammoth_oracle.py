"""CPU oracle for the routed encoder-decoder training step.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file; the
GPU library never does, and this file imports nothing from it.  Plain numpy, padded
[batch, length, d] arrays, float64 unless another dtype is requested, no blocking and no
fusion: every function is the textbook definition written out so it can be checked by eye.

What it follows
---------------
* Routing and gradient bookkeeping: paper section 3.2 (a task fixes an ordered set of
  modules; modules are position-specific; all tasks have the same number of modules) and
  Algorithm 1 (forward h_i = T_i(h_{i-1}) through the task's modules; a module not used by
  the task gets gradient 0; gradients are summed and divided by the number of uses n_j).
* Model sizes: paper section 4 (d=512, 8 heads, FFN 2048, position encoding).
* Everything the paper leaves open (pre-norm residual blocks, ReLU, sinusoidal positions,
  uniform label smoothing, Adam) is the reading fixed by the benchmark definition; each
  function below states its formula.

Pins (tests/test_oracle_*.py): central finite differences of the loss for every parameter
tensor; an independent autograd transcription built from library layer_norm / softmax /
cross_entropy / Adam; closed forms (ln V loss for equal logits, first Adam step, LayerNorm
moments, single-key attention); structural identities (split stack == whole stack,
zero adapter == no adapter, padding width, unused modules untouched).  Routed inference
(`forward_logits`, `greedy_decode`): the library transcription sentence by sentence, a greedy
loop written over it, the training step's own logits, prefix and batch-independence
properties, forced and forbidden EOS, equal top logits.  Beam search (`beam_decode`): beam 1
against the greedy search, a beam that holds every prefix against brute force over all sequences
scored with the library transcription, scores recomputed from it, carried finished hypotheses,
tie order.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PAD, BOS, EOS = 0, 1, 2
KINDS = ("src_emb", "enc", "tgt_emb", "dec", "gen", "adapter")
ALIGN = 64  # every tensor starts at a multiple of 64 elements inside its module's flat vector


# ----------------------------------------------------------------------------------------
# canonical per-module parameter layout
# ----------------------------------------------------------------------------------------
@dataclass(frozen=True)
class TensorSpec:
    name: str
    role: str  # "matrix" | "embed" | "bias" | "gamma" | "beta"
    shape: Tuple[int, ...]
    offset: int

    @property
    def size(self) -> int:
        return int(np.prod(self.shape))


def _round_up(n: int, a: int = ALIGN) -> int:
    return (n + a - 1) // a * a


def module_layout(kind: str, d: int, d_ff: int, vocab: int, n_layers: int = 0,
                  owns_final_norm: bool = False, adapter_dim: int = 0):
    """Tensor table of one module and the length of its flat vector.

    Order: embedding module E[V,d]; encoder layer ln1.g ln1.b Wq bq Wk bk Wv bv Wo bo ln2.g
    ln2.b W1 b1 W2 b2; decoder layer ln1, self-attention (8 tensors), ln2, cross-attention
    (8 tensors), ln3, W1 b1 W2 b2; a stack's closing lnf.g lnf.b if it owns the final norm;
    generator Wg[d,V] bg[V]; adapter layer ln.g ln.b Wd[d,r] bd[r] Wu[r,d] bu[d].
    Matrices are [in, out] row-major.  The flat length is rounded up to a multiple of 64.
    """
    specs: List[TensorSpec] = []
    cur = 0

    def add(name, role, shape):
        nonlocal cur
        cur = _round_up(cur)
        specs.append(TensorSpec(name, role, tuple(shape), cur))
        cur += int(np.prod(shape))

    def ln(prefix):
        add(prefix + ".g", "gamma", (d,))
        add(prefix + ".b", "beta", (d,))

    def attn(prefix):
        for p in ("q", "k", "v", "o"):
            add(f"{prefix}.W{p}", "matrix", (d, d))
            add(f"{prefix}.b{p}", "bias", (d,))

    def ffn(prefix):
        add(prefix + ".W1", "matrix", (d, d_ff))
        add(prefix + ".b1", "bias", (d_ff,))
        add(prefix + ".W2", "matrix", (d_ff, d))
        add(prefix + ".b2", "bias", (d,))

    if kind in ("src_emb", "tgt_emb"):
        add("E", "embed", (vocab, d))
    elif kind == "enc":
        for i in range(n_layers):
            ln(f"l{i}.ln1"); attn(f"l{i}.self"); ln(f"l{i}.ln2"); ffn(f"l{i}")
        if owns_final_norm:
            ln("lnf")
    elif kind == "dec":
        for i in range(n_layers):
            ln(f"l{i}.ln1"); attn(f"l{i}.self"); ln(f"l{i}.ln2"); attn(f"l{i}.cross")
            ln(f"l{i}.ln3"); ffn(f"l{i}")
        if owns_final_norm:
            ln("lnf")
    elif kind == "gen":
        add("Wg", "matrix", (d, vocab))
        add("bg", "bias", (vocab,))
    elif kind == "adapter":
        r = adapter_dim
        for i in range(n_layers):
            ln(f"l{i}.ln")
            add(f"l{i}.Wd", "matrix", (d, r)); add(f"l{i}.bd", "bias", (r,))
            add(f"l{i}.Wu", "matrix", (r, d)); add(f"l{i}.bu", "bias", (d,))
    else:
        raise ValueError(f"unknown module kind {kind!r}")
    return specs, _round_up(cur)


class _Module:
    def __init__(self, kind, name, position, n_layers, owns_final_norm, adapter_dim, stack,
                 specs, total, dtype):
        self.kind, self.name, self.position = kind, name, position
        self.n_layers, self.owns_final_norm = n_layers, owns_final_norm
        self.adapter_dim, self.stack = adapter_dim, stack
        self.specs, self.total = specs, total
        self.theta = np.zeros(total, dtype=dtype)
        self.grad = np.zeros(total, dtype=dtype)  # the module's gradient bucket
        self.m = np.zeros(total, dtype=dtype)
        self.v = np.zeros(total, dtype=dtype)
        self.t = 0          # Adam step count of this module
        self.touched = 0    # n_j: uses since the last update
        self._by_name = {s.name: s for s in specs}

    def p(self, name):
        s = self._by_name[name]
        return self.theta[s.offset:s.offset + s.size].reshape(s.shape)

    def g(self, name):
        s = self._by_name[name]
        return self.grad[s.offset:s.offset + s.size].reshape(s.shape)


# ----------------------------------------------------------------------------------------
# building blocks: each forward returns (output, cache); each backward consumes the cache
# ----------------------------------------------------------------------------------------
def positional_table(max_len: int, d: int) -> np.ndarray:
    """PE[p, 2k] = sin(p * 10000^(-2k/d)), PE[p, 2k+1] = cos(p * 10000^(-2k/d)), float64."""
    p = np.arange(max_len, dtype=np.float64)[:, None]
    k = np.arange(d // 2, dtype=np.float64)[None, :]
    ang = p * np.power(10000.0, -2.0 * k / d)
    pe = np.zeros((max_len, d), dtype=np.float64)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe


def layernorm_fwd(x, gamma, beta, eps):
    """y = gamma * (x - mean) / sqrt(biased var + eps) + beta over the last axis."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + x.dtype.type(eps))
    xhat = xc * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    """dx = rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)); dgamma, dbeta row sums."""
    xhat, rstd = cache
    dxhat = dy * gamma
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def linear_fwd(x, W, b):
    """y = x W + b with W [in, out]; leading axes of x are flattened to rows."""
    y = x.reshape(-1, W.shape[0]) @ W + b
    return y.reshape(x.shape[:-1] + (W.shape[1],))


def linear_bwd(dy, x, W):
    """dX = dY W^T, dW = X^T dY, db = sum over rows of dY."""
    d_in, d_out = W.shape
    dy2, x2 = dy.reshape(-1, d_out), x.reshape(-1, d_in)
    dx = (dy2 @ W.T).reshape(x.shape)
    dW = x2.T @ dy2
    db = dy2.sum(axis=0)
    return dx, dW, db


def _split_heads(x, H):
    B, L, d = x.shape
    return x.reshape(B, L, H, d // H).transpose(0, 2, 1, 3)  # [B,H,L,dh]


def _merge_heads(x):
    B, H, L, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B, L, H * dh)


def attention_fwd(xq, xkv, prm, blocked, H):
    """Multi-head attention: per head P = softmax(q k^T / sqrt(d_h)) with blocked keys at
    probability exactly 0, o = P v, output = concat(o) Wo + bo.
    xq [B,Lq,d] feeds the query projection, xkv [B,Lk,d] the key and value projections;
    blocked [B,Lq,Lk] is True where query i must not see key j."""
    Wq, bq, Wk, bk, Wv, bv, Wo, bo = prm
    q = _split_heads(linear_fwd(xq, Wq, bq), H)
    k = _split_heads(linear_fwd(xkv, Wk, bk), H)
    v = _split_heads(linear_fwd(xkv, Wv, bv), H)
    dh = q.shape[-1]
    scale = q.dtype.type(1.0 / np.sqrt(dh))
    s = (q @ k.transpose(0, 1, 3, 2)) * scale
    s = np.where(blocked[:, None, :, :], -np.inf, s)
    smax = s.max(axis=-1, keepdims=True)
    e = np.exp(s - smax)  # exp(-inf) = 0 exactly for blocked keys
    P = e / e.sum(axis=-1, keepdims=True)
    o = _merge_heads(P @ v)
    y = linear_fwd(o, Wo, bo)
    return y, (xq, xkv, q, k, v, P, o, scale)


def attention_bwd(dy, cache, prm, H):
    """dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(dP * P)) * scale, dQ = dS K,
    dK = dS^T Q, then the three input projections and the output projection transposed."""
    Wq, bq, Wk, bk, Wv, bv, Wo, bo = prm
    xq, xkv, q, k, v, P, o, scale = cache
    do, dWo, dbo = linear_bwd(dy, o, Wo)
    do = _split_heads(do, H)
    dv = P.transpose(0, 1, 3, 2) @ do
    dP = do @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True)) * scale
    dq = dS @ k
    dk = dS.transpose(0, 1, 3, 2) @ q
    dxq, dWq, dbq = linear_bwd(_merge_heads(dq), xq, Wq)
    dxk, dWk, dbk = linear_bwd(_merge_heads(dk), xkv, Wk)
    dxv, dWv, dbv = linear_bwd(_merge_heads(dv), xkv, Wv)
    return dxq, dxk + dxv, (dWq, dbq, dWk, dbk, dWv, dbv, dWo, dbo)


def ffn_fwd(x, W1, b1, W2, b2):
    """relu(x W1 + b1) W2 + b2 (also the adapter's bottleneck with W1=Wd, W2=Wu)."""
    pre = linear_fwd(x, W1, b1)
    hid = np.maximum(pre, 0)
    return linear_fwd(hid, W2, b2), (x, pre, hid)


def ffn_bwd(dy, cache, W1, W2):
    x, pre, hid = cache
    dhid, dW2, db2 = linear_bwd(dy, hid, W2)
    dpre = dhid * (pre > 0)  # strict: derivative 0 at pre == 0
    dx, dW1, db1 = linear_bwd(dpre, x, W1)
    return dx, (dW1, db1, dW2, db2)


def smoothed_ce(z, labels, eps_ls):
    """Per-row label-smoothed cross-entropy against q = (1-eps) onehot(y) + eps/V, and
    softmax(z) - q.  z [U,V], labels [U]."""
    U, V = z.shape
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax + np.log(np.exp(z - zmax).sum(axis=-1, keepdims=True))
    logp = z - lse
    eps_ls = z.dtype.type(eps_ls)
    nll = -logp[np.arange(U), labels]
    uni = -logp.sum(axis=-1) / V
    loss_rows = (1 - eps_ls) * nll + eps_ls * uni
    q = np.full_like(z, eps_ls / V)
    q[np.arange(U), labels] += 1 - eps_ls
    return loss_rows, np.exp(logp) - q


# ----------------------------------------------------------------------------------------
# the model: registry, routes, training step, update
# ----------------------------------------------------------------------------------------
class Oracle:
    def __init__(self, d_model, n_heads, d_ff, vocab, max_len, label_smoothing=0.1,
                 adam_beta1=0.9, adam_beta2=0.98, adam_eps=1e-9, ln_eps=1e-6,
                 dtype=np.float64, keep_trace=False):
        assert d_model % n_heads == 0 and d_model % 2 == 0
        self.d, self.H, self.F, self.V = d_model, n_heads, d_ff, vocab
        self.max_len = max_len
        self.eps_ls, self.b1, self.b2 = label_smoothing, adam_beta1, adam_beta2
        self.adam_eps, self.ln_eps = adam_eps, ln_eps
        self.dtype = np.dtype(dtype)
        self.pe = positional_table(max_len, d_model).astype(self.dtype)
        self.modules: List[_Module] = []
        self.routes: List[List[int]] = []
        self.keep_trace = keep_trace
        self.trace: Dict[str, object] = {}

    # ---- registry (section 3.2: position-specific modules, layers per position) ----------
    def register_module(self, kind, name="", position=0, n_layers=0, owns_final_norm=False,
                        adapter_dim=0, stack="", init: Optional[np.ndarray] = None,
                        shell: bool = False) -> int:
        specs, total = module_layout(kind, self.d, self.F, self.V, n_layers, owns_final_norm,
                                     adapter_dim)
        mod = _Module(kind, name, position, n_layers, owns_final_norm, adapter_dim, stack,
                      specs, 0 if shell else total, self.dtype)
        mod.total = total
        if init is not None:
            assert init.shape == (total,)
            mod.theta[:] = init
        self.modules.append(mod)
        return len(self.modules) - 1

    # ---- routes (a task = ordered module list; same count for every task) ----------------
    def parse_route(self, ids: Sequence[int]):
        """Splits src_emb, enc[0..], tgt_emb, dec[0..], gen, adapters... and checks that
        positions are consecutive and that exactly the last stack position closes the stack."""
        ids = [int(i) for i in ids]
        if any(i < 0 or i >= len(self.modules) for i in ids):
            raise ValueError("unknown module id in route")
        kinds = [self.modules[i].kind for i in ids]
        k = 0

        def take(kind, many):
            nonlocal k
            got = []
            while k < len(ids) and kinds[k] == kind:
                got.append(ids[k]); k += 1
                if not many:
                    break
            return got

        src, enc = take("src_emb", False), take("enc", True)
        tgt, dec = take("tgt_emb", False), take("dec", True)
        gen, ada = take("gen", False), take("adapter", True)
        if k != len(ids) or not (src and enc and tgt and dec and gen):
            raise ValueError("route must be src_emb, enc.., tgt_emb, dec.., gen, adapters..")
        for stack in (enc, dec):
            for pos, i in enumerate(stack):
                m = self.modules[i]
                if m.position != pos:
                    raise ValueError("module used at a position it was not defined for")
                if m.owns_final_norm != (pos == len(stack) - 1):
                    raise ValueError("exactly the last position of a stack owns the final norm")
        ad = {"enc": None, "dec": None}
        for i in ada:
            m = self.modules[i]
            if m.stack not in ad or ad[m.stack] is not None:
                raise ValueError("at most one adapter per stack")
            n_stack = sum(self.modules[j].n_layers for j in (enc if m.stack == "enc" else dec))
            if m.n_layers != n_stack:
                raise ValueError("adapter must cover every layer of its stack")
            ad[m.stack] = i
        if len(set(ids)) != len(ids):
            raise ValueError("a module may appear once in a route")
        return src[0], enc, tgt[0], dec, gen[0], ad

    def route_task(self, ids: Sequence[int]) -> int:
        self.parse_route(ids)
        if self.routes and len(self.routes[0]) != len(ids):
            raise ValueError("all tasks must involve the same number of modules")
        self.routes.append([int(i) for i in ids])
        return len(self.routes) - 1

    # ---- token bookkeeping -----------------------------------------------------------------
    @staticmethod
    def packed_view(src_ids, tgt_ids, lengths):
        """Row-by-row listing of the real (non-pad) positions, sentence after sentence:
        source token and position; decoder input token, label and position (decoder input =
        target without its last token, label = target shifted by one)."""
        src_ids, tgt_ids, lengths = map(np.asarray, (src_ids, tgt_ids, lengths))
        s_len, u_len = lengths[:, 0], lengths[:, 1] - 1
        out = dict(cu_s=np.concatenate([[0], np.cumsum(s_len)]).astype(np.int32),
                   cu_u=np.concatenate([[0], np.cumsum(u_len)]).astype(np.int32))
        out["src_tok"] = np.concatenate([src_ids[b, :s] for b, s in enumerate(s_len)])
        out["src_pos"] = np.concatenate([np.arange(s) for s in s_len]).astype(np.int32)
        out["dec_tok"] = np.concatenate([tgt_ids[b, :u] for b, u in enumerate(u_len)])
        out["label"] = np.concatenate([tgt_ids[b, 1:u + 1] for b, u in enumerate(u_len)])
        out["dec_pos"] = np.concatenate([np.arange(u) for u in u_len]).astype(np.int32)
        return out

    @staticmethod
    def check_batch(src_ids, tgt_ids, lengths, vocab, max_len):
        src_ids, tgt_ids, lengths = map(np.asarray, (src_ids, tgt_ids, lengths))
        B = len(lengths)
        assert src_ids.shape[0] == B and tgt_ids.shape[0] == B and B >= 1
        S_max, T_max = src_ids.shape[1], tgt_ids.shape[1]
        assert S_max <= max_len and T_max - 1 <= max_len
        for b in range(B):
            s, t = int(lengths[b, 0]), int(lengths[b, 1])
            assert 1 <= s <= S_max and 2 <= t <= T_max
            assert (src_ids[b, s:] == PAD).all() and (tgt_ids[b, t:] == PAD).all()
        assert src_ids.min() >= 0 and src_ids.max() < vocab
        assert tgt_ids.min() >= 0 and tgt_ids.max() < vocab

    # ---- layers ------------------------------------------------------------------------------
    def _attn_prm(self, m: _Module, prefix):
        return tuple(m.p(f"{prefix}.{n}") for n in ("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo"))

    def _attn_acc(self, m: _Module, prefix, grads):
        for n, g in zip(("Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo"), grads):
            m.g(f"{prefix}.{n}")[...] += g

    def _adapter_fwd(self, x, ad: _Module, li):
        a, c_ln = layernorm_fwd(x, ad.p(f"l{li}.ln.g"), ad.p(f"l{li}.ln.b"), self.ln_eps)
        y, c_f = ffn_fwd(a, ad.p(f"l{li}.Wd"), ad.p(f"l{li}.bd"), ad.p(f"l{li}.Wu"), ad.p(f"l{li}.bu"))
        return x + y, (c_ln, c_f)

    def _adapter_bwd(self, dx, cache, ad: _Module, li):
        c_ln, c_f = cache
        da, (dWd, dbd, dWu, dbu) = ffn_bwd(dx, c_f, ad.p(f"l{li}.Wd"), ad.p(f"l{li}.Wu"))
        for n, g in (("Wd", dWd), ("bd", dbd), ("Wu", dWu), ("bu", dbu)):
            ad.g(f"l{li}.{n}")[...] += g
        dln, dg, db = layernorm_bwd(da, c_ln, ad.p(f"l{li}.ln.g"))
        ad.g(f"l{li}.ln.g")[...] += dg
        ad.g(f"l{li}.ln.b")[...] += db
        return dx + dln

    def _enc_layer_fwd(self, x, m, i, blocked):
        a, c1 = layernorm_fwd(x, m.p(f"l{i}.ln1.g"), m.p(f"l{i}.ln1.b"), self.ln_eps)
        y, ca = attention_fwd(a, a, self._attn_prm(m, f"l{i}.self"), blocked, self.H)
        x = x + y
        f, c2 = layernorm_fwd(x, m.p(f"l{i}.ln2.g"), m.p(f"l{i}.ln2.b"), self.ln_eps)
        y, cf = ffn_fwd(f, m.p(f"l{i}.W1"), m.p(f"l{i}.b1"), m.p(f"l{i}.W2"), m.p(f"l{i}.b2"))
        return x + y, (c1, ca, c2, cf)

    def _enc_layer_bwd(self, dx, cache, m, i):
        c1, ca, c2, cf = cache
        df, (dW1, db1, dW2, db2) = ffn_bwd(dx, cf, m.p(f"l{i}.W1"), m.p(f"l{i}.W2"))
        for n, g in (("W1", dW1), ("b1", db1), ("W2", dW2), ("b2", db2)):
            m.g(f"l{i}.{n}")[...] += g
        dln, dg, db = layernorm_bwd(df, c2, m.p(f"l{i}.ln2.g"))
        m.g(f"l{i}.ln2.g")[...] += dg; m.g(f"l{i}.ln2.b")[...] += db
        dx = dx + dln
        dq_in, dkv_in, grads = attention_bwd(dx, ca, self._attn_prm(m, f"l{i}.self"), self.H)
        self._attn_acc(m, f"l{i}.self", grads)
        dln, dg, db = layernorm_bwd(dq_in + dkv_in, c1, m.p(f"l{i}.ln1.g"))
        m.g(f"l{i}.ln1.g")[...] += dg; m.g(f"l{i}.ln1.b")[...] += db
        return dx + dln

    def _dec_layer_fwd(self, x, mem, m, i, blocked_self, blocked_cross):
        a, c1 = layernorm_fwd(x, m.p(f"l{i}.ln1.g"), m.p(f"l{i}.ln1.b"), self.ln_eps)
        y, ca = attention_fwd(a, a, self._attn_prm(m, f"l{i}.self"), blocked_self, self.H)
        x = x + y
        c, c2 = layernorm_fwd(x, m.p(f"l{i}.ln2.g"), m.p(f"l{i}.ln2.b"), self.ln_eps)
        y, cc = attention_fwd(c, mem, self._attn_prm(m, f"l{i}.cross"), blocked_cross, self.H)
        x = x + y
        f, c3 = layernorm_fwd(x, m.p(f"l{i}.ln3.g"), m.p(f"l{i}.ln3.b"), self.ln_eps)
        y, cf = ffn_fwd(f, m.p(f"l{i}.W1"), m.p(f"l{i}.b1"), m.p(f"l{i}.W2"), m.p(f"l{i}.b2"))
        return x + y, (c1, ca, c2, cc, c3, cf)

    def _dec_layer_bwd(self, dx, dmem, cache, m, i):
        c1, ca, c2, cc, c3, cf = cache
        df, (dW1, db1, dW2, db2) = ffn_bwd(dx, cf, m.p(f"l{i}.W1"), m.p(f"l{i}.W2"))
        for n, g in (("W1", dW1), ("b1", db1), ("W2", dW2), ("b2", db2)):
            m.g(f"l{i}.{n}")[...] += g
        dln, dg, db = layernorm_bwd(df, c3, m.p(f"l{i}.ln3.g"))
        m.g(f"l{i}.ln3.g")[...] += dg; m.g(f"l{i}.ln3.b")[...] += db
        dx = dx + dln
        dq_in, dkv_in, grads = attention_bwd(dx, cc, self._attn_prm(m, f"l{i}.cross"), self.H)
        self._attn_acc(m, f"l{i}.cross", grads)
        dmem = dmem + dkv_in
        dln, dg, db = layernorm_bwd(dq_in, c2, m.p(f"l{i}.ln2.g"))
        m.g(f"l{i}.ln2.g")[...] += dg; m.g(f"l{i}.ln2.b")[...] += db
        dx = dx + dln
        dq_in, dkv_in, grads = attention_bwd(dx, ca, self._attn_prm(m, f"l{i}.self"), self.H)
        self._attn_acc(m, f"l{i}.self", grads)
        dln, dg, db = layernorm_bwd(dq_in + dkv_in, c1, m.p(f"l{i}.ln1.g"))
        m.g(f"l{i}.ln1.g")[...] += dg; m.g(f"l{i}.ln1.b")[...] += db
        return dx + dln, dmem

    # ---- one training step of one task (Algorithm 1, forward and backward parts) ----------
    def train_step(self, task: int, src_ids, tgt_ids, lengths) -> float:
        src_ids, tgt_ids, lengths = (np.asarray(a) for a in (src_ids, tgt_ids, lengths))
        self.check_batch(src_ids, tgt_ids, lengths, self.V, self.max_len)
        i_src, enc_ids, i_tgt, dec_ids, i_gen, ad = self.parse_route(self.routes[task])
        M = self.modules
        dt = self.dtype.type
        B, S_max = src_ids.shape
        U_max = tgt_ids.shape[1] - 1
        s_len, u_len = lengths[:, 0], lengths[:, 1] - 1
        dec_in, labels = tgt_ids[:, :-1], tgt_ids[:, 1:]
        src_real = np.arange(S_max)[None, :] < s_len[:, None]        # [B,S_max]
        dec_real = np.arange(U_max)[None, :] < u_len[:, None]        # [B,U_max]
        U = int(u_len.sum())

        # who must not see whom
        enc_blocked = np.broadcast_to(~src_real[:, None, :], (B, S_max, S_max))
        causal = np.arange(U_max)[None, :] > np.arange(U_max)[:, None]
        dec_blocked = causal[None, :, :] | ~dec_real[:, None, :]
        cross_blocked = np.broadcast_to(~src_real[:, None, :], (B, U_max, S_max))

        for j in self.routes[task]:      # ready_T of Algorithm 1, kept as a use count
            M[j].touched += 1

        # ---------------- forward: h_i = T_i(h_{i-1}) over the task's modules ----------------
        sqrt_d = dt(np.sqrt(self.d))
        x = sqrt_d * M[i_src].p("E")[src_ids] + self.pe[None, :S_max, :]
        x = x * src_real[:, :, None]
        enc_caches, li = [], 0
        ad_e = M[ad["enc"]] if ad["enc"] is not None else None
        for j in enc_ids:
            for i in range(M[j].n_layers):
                x, c = self._enc_layer_fwd(x, M[j], i, enc_blocked)
                ca = None
                if ad_e is not None:
                    x, ca = self._adapter_fwd(x, ad_e, li)
                enc_caches.append((j, i, li, c, ca)); li += 1
        m_last = M[enc_ids[-1]]
        mem, c_encf = layernorm_fwd(x, m_last.p("lnf.g"), m_last.p("lnf.b"), self.ln_eps)

        y = sqrt_d * M[i_tgt].p("E")[dec_in] + self.pe[None, :U_max, :]
        y = y * dec_real[:, :, None]
        dec_caches, li = [], 0
        ad_d = M[ad["dec"]] if ad["dec"] is not None else None
        for j in dec_ids:
            for i in range(M[j].n_layers):
                y, c = self._dec_layer_fwd(y, mem, M[j], i, dec_blocked, cross_blocked)
                ca = None
                if ad_d is not None:
                    y, ca = self._adapter_fwd(y, ad_d, li)
                dec_caches.append((j, i, li, c, ca)); li += 1
        d_last = M[dec_ids[-1]]
        h, c_decf = layernorm_fwd(y, d_last.p("lnf.g"), d_last.p("lnf.b"), self.ln_eps)

        # ---------------- loss over the U real decoder positions -----------------------------
        h_real = h[dec_real]                       # [U,d], sentence after sentence
        y_real = labels[dec_real]
        z = linear_fwd(h_real, M[i_gen].p("Wg"), M[i_gen].p("bg"))
        loss_rows, p_minus_q = smoothed_ce(z, y_real, self.eps_ls)
        loss = loss_rows.sum() / dt(U)
        if self.keep_trace:
            self.trace = dict(loss_rows=loss_rows.copy(), src_real=src_real, dec_real=dec_real,
                              enc_blocked=enc_blocked, dec_blocked=dec_blocked,
                              cross_blocked=cross_blocked, logits=z.copy(), mem=mem.copy(),
                              enc_P=[c[3][1][5] for c in enc_caches],
                              dec_self_P=[c[3][1][5] for c in dec_caches],
                              dec_cross_P=[c[3][3][5] for c in dec_caches])

        # ---------------- backward (gradient of the loss; used modules only) -----------------
        dz = p_minus_q / dt(U)
        dh_real, dWg, dbg = linear_bwd(dz, h_real, M[i_gen].p("Wg"))
        M[i_gen].g("Wg")[...] += dWg
        M[i_gen].g("bg")[...] += dbg
        dh = np.zeros_like(h)
        dh[dec_real] = dh_real
        dy, dg, db = layernorm_bwd(dh, c_decf, d_last.p("lnf.g"))
        d_last.g("lnf.g")[...] += dg; d_last.g("lnf.b")[...] += db
        dmem = np.zeros_like(mem)
        for j, i, li, c, ca in reversed(dec_caches):
            if ca is not None:
                dy = self._adapter_bwd(dy, ca, ad_d, li)
            dy, dmem = self._dec_layer_bwd(dy, dmem, c, M[j], i)
        dE = M[i_tgt].g("E")
        np.add.at(dE, dec_in[dec_real], sqrt_d * dy[dec_real])

        dx, dg, db = layernorm_bwd(dmem, c_encf, m_last.p("lnf.g"))
        m_last.g("lnf.g")[...] += dg; m_last.g("lnf.b")[...] += db
        for j, i, li, c, ca in reversed(enc_caches):
            if ca is not None:
                dx = self._adapter_bwd(dx, ca, ad_e, li)
            dx = self._enc_layer_bwd(dx, c, M[j], i)
        dE = M[i_src].g("E")
        np.add.at(dE, src_ids[src_real], sqrt_d * dx[src_real])
        if self.keep_trace:
            self.trace["dx_src"], self.trace["dy_tgt"] = dx, dy
        return float(loss)

    # ---- routed inference (section 3.2: translating a task needs only that task's modules) ---
    def forward_logits(self, task: int, src_ids, src_len, dec_in, dec_len):
        """Generator logits [B, U_max, V] of one task for given decoder inputs: the forward half
        of `train_step` on its own (same modules in the same order, same masks), with nothing
        cached and no bookkeeping touched.  Rows at or beyond dec_len[b] are meaningless."""
        src_ids, dec_in = np.asarray(src_ids), np.asarray(dec_in)
        s_len, u_len = np.asarray(src_len), np.asarray(dec_len)
        i_src, enc_ids, i_tgt, dec_ids, i_gen, ad = self.parse_route(self.routes[task])
        M = self.modules
        dt = self.dtype.type
        B, S_max = src_ids.shape
        U_max = dec_in.shape[1]
        src_real = np.arange(S_max)[None, :] < s_len[:, None]
        dec_real = np.arange(U_max)[None, :] < u_len[:, None]
        enc_blocked = np.broadcast_to(~src_real[:, None, :], (B, S_max, S_max))
        causal = np.arange(U_max)[None, :] > np.arange(U_max)[:, None]
        dec_blocked = causal[None, :, :] | ~dec_real[:, None, :]
        cross_blocked = np.broadcast_to(~src_real[:, None, :], (B, U_max, S_max))

        sqrt_d = dt(np.sqrt(self.d))
        x = (sqrt_d * M[i_src].p("E")[src_ids] + self.pe[None, :S_max, :]) * src_real[:, :, None]
        ad_e = M[ad["enc"]] if ad["enc"] is not None else None
        li = 0
        for j in enc_ids:
            for i in range(M[j].n_layers):
                x, _ = self._enc_layer_fwd(x, M[j], i, enc_blocked)
                if ad_e is not None:
                    x, _ = self._adapter_fwd(x, ad_e, li)
                li += 1
        m_last = M[enc_ids[-1]]
        mem, _ = layernorm_fwd(x, m_last.p("lnf.g"), m_last.p("lnf.b"), self.ln_eps)

        y = (sqrt_d * M[i_tgt].p("E")[dec_in] + self.pe[None, :U_max, :]) * dec_real[:, :, None]
        ad_d = M[ad["dec"]] if ad["dec"] is not None else None
        li = 0
        for j in dec_ids:
            for i in range(M[j].n_layers):
                y, _ = self._dec_layer_fwd(y, mem, M[j], i, dec_blocked, cross_blocked)
                if ad_d is not None:
                    y, _ = self._adapter_fwd(y, ad_d, li)
                li += 1
        d_last = M[dec_ids[-1]]
        h, _ = layernorm_fwd(y, d_last.p("lnf.g"), d_last.p("lnf.b"), self.ln_eps)
        return linear_fwd(h, M[i_gen].p("Wg"), M[i_gen].p("bg"))

    def greedy_decode(self, task: int, src_ids, src_len, max_new: int):
        """Greedy translation, the slow way: for t = 0, 1, ... every sentence's decoder input is
        BOS followed by the t tokens it has produced, the whole model is run again from the
        source, and token t is the position-t logit row's largest entry (lowest index among
        equal ones).  A sentence stops once it has produced EOS (EOS is kept, PAD follows);
        it also stops after max_new tokens.  Returns (ids [B, max_new], produced counts [B]).
        The paper fixes no search procedure; this is the plainest one and is the reading the
        GPU path is held to."""
        src_ids, s_len = np.asarray(src_ids), np.asarray(src_len)
        B = src_ids.shape[0]
        assert 1 <= max_new <= self.max_len
        out = np.full((B, max_new), PAD, dtype=np.int32)
        n_out = np.zeros(B, dtype=np.int32)
        alive = np.ones(B, dtype=bool)
        for t in range(max_new):
            if not alive.any():
                break
            dec_in = np.concatenate([np.full((B, 1), BOS, dtype=np.int32), out[:, :t]], axis=1)
            # a finished sentence keeps its shorter input; its later rows are never looked at
            dec_len = np.where(alive, t + 1, np.maximum(n_out, 1)).astype(np.int32)
            z = self.forward_logits(task, src_ids, s_len, dec_in, dec_len)
            for b in range(B):
                if alive[b]:
                    tok = int(np.argmax(z[b, t]))       # numpy returns the first maximum
                    out[b, t] = tok
                    n_out[b] = t + 1
                    if tok == EOS:
                        alive[b] = False
        return out, n_out

    def beam_decode(self, task: int, src_ids, src_len, max_new: int, beam: int):
        """Beam search, the slow way (the paper fixes no search procedure; reading: the textbook
        length-synchronous beam with summed log-probabilities and no length normalisation).
        Per sentence a beam of at most `beam` hypotheses, best first, starting from the empty
        one with score 0.  Each step every unfinished hypothesis i is extended by every token v
        at score_i + log softmax(z_i)[v], where z_i is the generator's logit row after BOS and
        the hypothesis' tokens (the whole model is run again from the source); a finished
        hypothesis (one that ends in EOS) is carried over unchanged.  The `beam` best candidates
        form the next beam; ties go to the lower hypothesis index, then the lower token id.  The
        search ends when every hypothesis in the beam is finished or after max_new tokens; the
        first hypothesis is the result.  beam = 1 is `greedy_decode`.
        Returns (ids [B, max_new] padded with PAD, produced counts [B], scores [B])."""
        src_ids, s_len = np.asarray(src_ids), np.asarray(src_len)
        B = src_ids.shape[0]
        assert 1 <= max_new <= self.max_len and beam >= 1
        out = np.full((B, max_new), PAD, dtype=np.int32)
        n_out = np.zeros(B, dtype=np.int32)
        best = np.zeros(B, dtype=np.float64)
        for b in range(B):
            hyps = [([], 0.0, False)]                      # (tokens, score, finished)
            for t in range(max_new):
                live = [i for i, h in enumerate(hyps) if not h[2]]
                if not live:
                    break
                dec_in = np.full((len(live), t + 1), PAD, dtype=np.int32)
                dec_in[:, 0] = BOS
                for r, i in enumerate(live):
                    dec_in[r, 1:] = hyps[i][0]             # an unfinished hypothesis has exactly t tokens
                z = self.forward_logits(task, np.repeat(src_ids[b:b + 1], len(live), axis=0),
                                        np.repeat(s_len[b:b + 1], len(live)), dec_in,
                                        np.full(len(live), t + 1, dtype=np.int32))
                cand = []                                   # (-score, hypothesis index, token or -1)
                for i, h in enumerate(hyps):
                    if h[2]:
                        cand.append((-h[1], i, -1))
                for r, i in enumerate(live):
                    row = z[r, t].astype(np.float64)
                    mx = row.max()
                    logp = row - (mx + np.log(np.exp(row - mx).sum()))
                    for v in range(self.V):
                        cand.append((-(hyps[i][1] + logp[v]), i, v))
                cand.sort()
                nxt = []
                for neg, i, v in cand[:beam]:
                    toks, _, fin = hyps[i]
                    nxt.append((toks, -neg, True) if v < 0 else (toks + [v], -neg, v == EOS))
                hyps = nxt
            toks, score, _ = hyps[0]
            out[b, :len(toks)] = toks
            n_out[b] = len(toks)
            best[b] = score
        return out, n_out, best

    # ---- renormalise and update (Algorithm 1 last line + Adam) ---------------------------
    def apply_update(self, module_ids: Optional[Sequence[int]], lr: float):
        """For each requested module with n_j > 0: g = bucket / n_j, then one Adam step
        (bias-corrected, eps outside the square root, no weight decay), bucket and n_j reset.
        Modules with n_j = 0 are left exactly as they are."""
        ids = range(len(self.modules)) if module_ids is None else module_ids
        dt = self.dtype.type
        for j in ids:
            m = self.modules[int(j)]
            if m.touched == 0:
                continue
            g = m.grad / dt(m.touched)
            m.t += 1
            m.m[:] = dt(self.b1) * m.m + dt(1 - self.b1) * g
            m.v[:] = dt(self.b2) * m.v + dt(1 - self.b2) * g * g
            mhat = m.m / dt(1 - self.b1 ** m.t)
            vhat = m.v / dt(1 - self.b2 ** m.t)
            m.theta[:] = m.theta - dt(lr) * mhat / (np.sqrt(vhat) + dt(self.adam_eps))
            m.grad[:] = 0
            m.touched = 0


def build_from_setup(setup, dtype=np.float64, perturbed=False, keep_trace=False,
                     fill_params=None, needed=None):
    """Registers a set-up's modules and tasks; `fill_params` is the seeded initialiser
    (role, offset, size table -> float32 vector) passed in by the caller.  `needed`: optional set
    of module indices to materialise; the others are registered as empty shells (same ids and
    routes, no arrays) so that a large set-up can be checked one task at a time."""
    sh = setup.shape
    orc = Oracle(sh.d_model, sh.n_heads, sh.d_ff, sh.vocab, sh.max_len, sh.label_smoothing,
                 sh.adam_beta1, sh.adam_beta2, sh.adam_eps, sh.ln_eps, dtype=dtype,
                 keep_trace=keep_trace)
    for k, ms in enumerate(setup.modules):
        specs, total = module_layout(ms.kind, sh.d_model, sh.d_ff, sh.vocab, ms.n_layers,
                                     ms.owns_final_norm, ms.adapter_dim)
        init = None
        if needed is not None and k not in needed:
            j = orc.register_module(ms.kind, ms.name, ms.position, ms.n_layers, ms.owns_final_norm,
                                    ms.adapter_dim, ms.stack, None, shell=True)
            continue
        if fill_params is not None:
            init = fill_params([(s.role, s.offset, s.size) for s in specs], total,
                               setup.weight_seed * 1000 + k, perturbed).astype(dtype)
        orc.register_module(ms.kind, ms.name, ms.position, ms.n_layers, ms.owns_final_norm,
                            ms.adapter_dim, ms.stack, init)
    for _, ids in setup.tasks:
        orc.route_task(ids)
    return orc
