"""ctypes binding of libmammoth_hip.so: argument marshalling only, same names as the C ABI.

Every step of the training path runs inside the library's HIP kernels; nothing here computes.
The library must have been built (`python -m paper_2403_07544_amd.build`); a missing library is
an error, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmammoth_hip.so")

MM_OK, MM_EINVAL, MM_ENOMEM, MM_ESTATE, MM_ERANGE, MM_ENONFINITE, MM_EHIP = 0, -1, -2, -3, -4, -5, -6
STATUS_NAMES = {0: "MM_OK", -1: "MM_EINVAL", -2: "MM_ENOMEM", -3: "MM_ESTATE", -4: "MM_ERANGE",
                -5: "MM_ENONFINITE", -6: "MM_EHIP"}
MM_F32, MM_BF16 = 0, 1
KIND = {"src_emb": 0, "enc": 1, "tgt_emb": 2, "dec": 3, "gen": 4, "adapter": 5}
MM_HOST, MM_DEVICE = 0, 1
ROLE_NAMES = ("matrix", "embed", "bias", "gamma", "beta")
DUMP = {"cu_src": 0, "cu_dec": 1, "src_tok": 2, "src_pos": 3, "dec_tok": 4, "dec_pos": 5, "label": 6,
        "mask_enc": 7, "mask_dec": 8, "mask_cross": 9}
KERNEL_CLASSES = ("gemm", "attn_fwd", "attn_bwd", "layernorm_fwd", "layernorm_bwd", "embed",
                  "embed_grad", "ce", "colsum", "adam", "other")

EXPORTS = ("mm_create", "mm_destroy", "mm_register_module", "mm_route_task", "mm_train_step", "mm_translate_greedy", "mm_translate_beam",
           "mm_last_loss", "mm_apply_update", "mm_apply_update_noalloc", "mm_num_modules", "mm_get_route", "mm_get_touched",
           "mm_get_layout", "mm_get_params", "mm_set_params", "mm_get_grads", "mm_get_bucket_memory", "mm_set_grads",
           "mm_get_adam", "mm_get_working", "mm_debug_dump", "mm_debug_attention", "mm_profile", "mm_profile_read",
           "mm_last_error")


class MMConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("dtype", C.c_int32), ("label_smoothing", C.c_float), ("adam_beta1", C.c_float),
                ("adam_beta2", C.c_float), ("adam_eps", C.c_float), ("ln_eps", C.c_float),
                ("max_len", C.c_int32), ("max_batch_tokens", C.c_int32), ("hip_stream", C.c_void_p),
                ("plan_only", C.c_int32)]


class MMModuleDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("position", C.c_int32), ("n_layers", C.c_int32),
                ("owns_final_norm", C.c_int32), ("adapter_dim", C.c_int32), ("adapter_stack", C.c_int32),
                ("name", C.c_char_p)]


class MMError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load_library() -> C.CDLL:
    """Loads the built library; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2403_07544_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    pi32, pi64, pf32 = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float)
    sig = {
        "mm_create": [C.POINTER(MMConfig), C.POINTER(vp)],
        "mm_destroy": [vp],
        "mm_register_module": [vp, C.POINTER(MMModuleDesc), vp, i64, pi32],
        "mm_route_task": [vp, vp, i32, pi32],
        "mm_train_step": [vp, i32, vp, vp, vp, i32, i32, i32, i32, pf32],
        "mm_translate_greedy": [vp, i32, vp, vp, i32, i32, i32, i32, vp, vp],
        "mm_translate_beam": [vp, i32, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp],
        "mm_last_loss": [vp, pf32],
        "mm_apply_update": [vp, vp, i32, f32],
        "mm_apply_update_noalloc": [vp, vp, i32, f32],
        "mm_num_modules": [vp, pi32],
        "mm_get_route": [vp, i32, vp, pi32],
        "mm_get_touched": [vp, vp, i32],
        "mm_get_layout": [vp, i32, vp, vp, vp, vp, pi32, pi64],
        "mm_get_params": [vp, i32, vp, i64],
        "mm_set_params": [vp, i32, vp, i64],
        "mm_get_grads": [vp, i32, vp, i64],
        "mm_get_bucket_memory": [vp, i32, vp, i64],
        "mm_set_grads": [vp, i32, vp, i64, i32],
        "mm_get_adam": [vp, i32, vp, vp, i64, pi64],
        "mm_get_working": [vp, i32, vp, i64],
        "mm_debug_dump": [vp, i32, vp, pi64],
        "mm_debug_attention": [vp, i32, i32, vp, pi64],
        "mm_profile": [vp, i32],
        "mm_profile_read": [vp, vp, vp, vp],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.mm_last_error.argtypes = [vp]
    lib.mm_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Context:
    """One GPU, one stream, one model shape.  Methods mirror the C entry points."""

    def __init__(self, d_model, n_heads, d_ff, vocab, dtype="bf16", max_len=100, max_batch_tokens=8192,
                 label_smoothing=0.1, adam_beta1=0.9, adam_beta2=0.98, adam_eps=1e-9, ln_eps=1e-6,
                 hip_stream: int = 0, plan_only: bool = False):
        self.lib = load_library()
        self.cfg = MMConfig(d_model, n_heads, d_ff, vocab, MM_BF16 if dtype == "bf16" else MM_F32,
                            label_smoothing, adam_beta1, adam_beta2, adam_eps, ln_eps, max_len,
                            max_batch_tokens, hip_stream or None, 1 if plan_only else 0)
        self.handle = C.c_void_p()
        st = self.lib.mm_create(C.byref(self.cfg), C.byref(self.handle))
        if st != MM_OK:
            msg = self.lib.mm_last_error(self.handle).decode() if self.handle else "mm_create rejected the configuration"
            if self.handle:
                self.lib.mm_destroy(self.handle)
                self.handle = C.c_void_p()
            raise MMError(st, msg)

    # -- plumbing ---------------------------------------------------------------------------------
    def _check(self, st: int):
        if st != MM_OK:
            raise MMError(st, self.lib.mm_last_error(self.handle).decode())

    def close(self):
        if getattr(self, "handle", None):
            self.lib.mm_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- registry and routes ----------------------------------------------------------------------
    def mm_register_module(self, kind: str, name: str = "", position: int = 0, n_layers: int = 0,
                           owns_final_norm: bool = False, adapter_dim: int = 0, stack: str = "",
                           init: Optional[np.ndarray] = None) -> int:
        desc = MMModuleDesc(KIND[kind], position, n_layers, int(owns_final_norm), adapter_dim,
                            1 if stack == "dec" else 0, name.encode())
        out = C.c_int32(-1)
        n = 0
        if init is not None:
            init = np.ascontiguousarray(init, dtype=np.float32)
            n = init.size
        self._check(self.lib.mm_register_module(self.handle, C.byref(desc), _ptr(init), n, C.byref(out)))
        return out.value

    def mm_route_task(self, module_ids: Sequence[int]) -> int:
        ids = np.ascontiguousarray(module_ids, dtype=np.int32)
        out = C.c_int32(-1)
        self._check(self.lib.mm_route_task(self.handle, _ptr(ids), len(ids), C.byref(out)))
        return out.value

    # -- the hot path -----------------------------------------------------------------------------
    def mm_train_step(self, task: int, src_ids, tgt_ids, lengths, sync: bool = True) -> Optional[float]:
        """src_ids/tgt_ids: numpy int32 arrays (host) or torch int32 CUDA tensors (device)."""
        lengths = np.ascontiguousarray(lengths, dtype=np.int32)
        B = lengths.shape[0]
        if isinstance(src_ids, np.ndarray):
            src = np.ascontiguousarray(src_ids, dtype=np.int32)
            tgt = np.ascontiguousarray(tgt_ids, dtype=np.int32)
            sp, tp, mem = _ptr(src), _ptr(tgt), MM_HOST
        else:  # torch tensors on the GPU: only their addresses are used
            assert src_ids.is_cuda and tgt_ids.is_cuda and src_ids.is_contiguous() and tgt_ids.is_contiguous()
            assert str(src_ids.dtype) == "torch.int32" and str(tgt_ids.dtype) == "torch.int32"
            src, tgt = src_ids, tgt_ids
            sp, tp, mem = C.c_void_p(src.data_ptr()), C.c_void_p(tgt.data_ptr()), MM_DEVICE
        assert src.shape[0] == B and tgt.shape[0] == B
        loss = C.c_float(0.0)
        st = self.lib.mm_train_step(self.handle, task, sp, tp, _ptr(lengths), B, src.shape[1], tgt.shape[1],
                                    mem, C.byref(loss) if sync else None)
        self._check(st)
        return loss.value if sync else None

    def mm_translate_greedy(self, task: int, src_ids, src_lengths, max_new: int):
        """src_ids: numpy int32 array (host) or torch int32 CUDA tensor.  Returns (ids [B, max_new],
        produced counts [B]) as numpy int32 arrays."""
        src_lengths = np.ascontiguousarray(src_lengths, dtype=np.int32)
        B = src_lengths.shape[0]
        if isinstance(src_ids, np.ndarray):
            src = np.ascontiguousarray(src_ids, dtype=np.int32)
            sp, mem = _ptr(src), MM_HOST
        else:
            assert src_ids.is_cuda and src_ids.is_contiguous() and str(src_ids.dtype) == "torch.int32"
            src = src_ids
            sp, mem = C.c_void_p(src.data_ptr()), MM_DEVICE
        assert src.shape[0] == B
        out_ids = np.zeros((B, max(int(max_new), 0)), dtype=np.int32)
        out_len = np.zeros(B, dtype=np.int32)
        st = self.lib.mm_translate_greedy(self.handle, task, sp, _ptr(src_lengths), B, src.shape[1], int(max_new),
                                          mem, _ptr(out_ids), _ptr(out_len))
        self._check(st)
        return out_ids, out_len

    def mm_translate_beam(self, task: int, src_ids, src_lengths, max_new: int, beam: int):
        """As mm_translate_greedy, with a beam of `beam` hypotheses per sentence.  Returns (ids
        [B, max_new], produced counts [B], summed log-probabilities [B] float32)."""
        src_lengths = np.ascontiguousarray(src_lengths, dtype=np.int32)
        B = src_lengths.shape[0]
        if isinstance(src_ids, np.ndarray):
            src = np.ascontiguousarray(src_ids, dtype=np.int32)
            sp, mem = _ptr(src), MM_HOST
        else:
            assert src_ids.is_cuda and src_ids.is_contiguous() and str(src_ids.dtype) == "torch.int32"
            src = src_ids
            sp, mem = C.c_void_p(src.data_ptr()), MM_DEVICE
        assert src.shape[0] == B
        out_ids = np.zeros((B, max(int(max_new), 0)), dtype=np.int32)
        out_len = np.zeros(B, dtype=np.int32)
        out_score = np.zeros(B, dtype=np.float32)
        st = self.lib.mm_translate_beam(self.handle, task, sp, _ptr(src_lengths), B, src.shape[1], int(max_new),
                                        int(beam), mem, _ptr(out_ids), _ptr(out_len), _ptr(out_score))
        self._check(st)
        return out_ids, out_len, out_score

    def mm_last_loss(self) -> float:
        loss = C.c_float(0.0)
        self._check(self.lib.mm_last_loss(self.handle, C.byref(loss)))
        return loss.value

    def mm_apply_update(self, module_ids: Optional[Sequence[int]], lr: float):
        if module_ids is None:
            self._check(self.lib.mm_apply_update(self.handle, None, 0, lr))
        else:
            ids = np.ascontiguousarray(module_ids, dtype=np.int32)
            self._check(self.lib.mm_apply_update(self.handle, _ptr(ids), len(ids), lr))

    def mm_apply_update_noalloc(self, module_ids: Optional[Sequence[int]], lr: float):
        if module_ids is None:
            self._check(self.lib.mm_apply_update_noalloc(self.handle, None, 0, lr))
        else:
            ids = np.ascontiguousarray(module_ids, dtype=np.int32)
            self._check(self.lib.mm_apply_update_noalloc(self.handle, _ptr(ids), len(ids), lr))

    # -- introspection ----------------------------------------------------------------------------
    def mm_num_modules(self) -> int:
        n = C.c_int32(0)
        self._check(self.lib.mm_num_modules(self.handle, C.byref(n)))
        return n.value

    def mm_get_route(self, task: int) -> List[int]:
        n = C.c_int32(256)
        ids = np.zeros(256, dtype=np.int32)
        self._check(self.lib.mm_get_route(self.handle, task, _ptr(ids), C.byref(n)))
        return ids[:n.value].tolist()

    def mm_get_touched(self) -> np.ndarray:
        n = self.mm_num_modules()
        out = np.zeros(max(n, 1), dtype=np.int32)
        self._check(self.lib.mm_get_touched(self.handle, _ptr(out), len(out)))
        return out[:n]

    def mm_get_layout(self, module: int) -> Tuple[List[Tuple[str, int, int, int]], int]:
        """[(role, offset, rows, cols)], bucket length."""
        n = C.c_int32(0)
        total = C.c_int64(0)
        self._check(self.lib.mm_get_layout(self.handle, module, None, None, None, None, C.byref(n), C.byref(total)))
        k = n.value
        off = np.zeros(k, dtype=np.int64)
        rows, cols, roles = (np.zeros(k, dtype=np.int32) for _ in range(3))
        self._check(self.lib.mm_get_layout(self.handle, module, _ptr(off), _ptr(rows), _ptr(cols), _ptr(roles),
                                           C.byref(n), C.byref(total)))
        return [(ROLE_NAMES[roles[i]], int(off[i]), int(rows[i]), int(cols[i])) for i in range(k)], total.value

    def _bucket_len(self, module: int) -> int:
        return self.mm_get_layout(module)[1]

    def _get(self, fn, module: int) -> np.ndarray:
        out = np.zeros(self._bucket_len(module), dtype=np.float32)
        self._check(fn(self.handle, module, _ptr(out), out.size))
        return out

    def mm_get_params(self, module: int) -> np.ndarray:
        return self._get(self.lib.mm_get_params, module)

    def mm_get_grads(self, module: int) -> np.ndarray:
        return self._get(self.lib.mm_get_grads, module)

    def mm_get_bucket_memory(self, module: int) -> np.ndarray:
        return self._get(self.lib.mm_get_bucket_memory, module)

    def mm_get_working(self, module: int) -> np.ndarray:
        return self._get(self.lib.mm_get_working, module)

    def mm_set_params(self, module: int, values: np.ndarray):
        v = np.ascontiguousarray(values, dtype=np.float32)
        self._check(self.lib.mm_set_params(self.handle, module, _ptr(v), v.size))

    def mm_set_grads(self, module: int, values: np.ndarray, n_uses: int):
        v = np.ascontiguousarray(values, dtype=np.float32)
        self._check(self.lib.mm_set_grads(self.handle, module, _ptr(v), v.size, n_uses))

    def mm_get_adam(self, module: int):
        n = self._bucket_len(module)
        m, v = np.zeros(n, dtype=np.float32), np.zeros(n, dtype=np.float32)
        t = C.c_int64(0)
        self._check(self.lib.mm_get_adam(self.handle, module, _ptr(m), _ptr(v), n, C.byref(t)))
        return m, v, t.value

    def mm_debug_dump(self, what: str) -> np.ndarray:
        code = DUMP[what]
        nbytes = C.c_int64(0)
        self._check(self.lib.mm_debug_dump(self.handle, code, None, C.byref(nbytes)))
        dtype = np.uint8 if what.startswith("mask") else np.int32
        out = np.zeros(nbytes.value // np.dtype(dtype).itemsize, dtype=dtype)
        self._check(self.lib.mm_debug_dump(self.handle, code, _ptr(out), C.byref(nbytes)))
        return out

    def mm_debug_attention(self, kind: str, layer: int, B: int, H: int) -> np.ndarray:
        """Probabilities [B, H, Lq, Lk] of one attention block of the last step, read off the
        step's own forward attention kernel.  kind: 'enc', 'dec_self' or 'dec_cross'."""
        code = {"enc": 0, "dec_self": 1, "dec_cross": 2}[kind]
        n = C.c_int64(0)
        self._check(self.lib.mm_debug_attention(self.handle, code, layer, None, C.byref(n)))
        out = np.zeros(n.value, dtype=np.float32)
        self._check(self.lib.mm_debug_attention(self.handle, code, layer, _ptr(out), C.byref(n)))
        return out.reshape(B, H, -1)

    def mm_profile(self, enable: bool):
        self._check(self.lib.mm_profile(self.handle, 1 if enable else 0))

    def mm_profile_read(self):
        k = len(KERNEL_CLASSES)
        ms, work = np.zeros(k, dtype=np.float64), np.zeros(k, dtype=np.float64)
        n = np.zeros(k, dtype=np.int64)
        self._check(self.lib.mm_profile_read(self.handle, _ptr(ms), _ptr(n), _ptr(work)))
        return {name: dict(ms=float(ms[i]), launches=int(n[i]), work=float(work[i]))
                for i, name in enumerate(KERNEL_CLASSES)}


def context_from_setup(setup, fill_params=None, perturbed=False, plan_only=False, hip_stream=0,
                       max_batch_tokens=None) -> Context:
    """Creates a context for one of the synthetic set-ups, registers its modules (initial values
    drawn by `fill_params` from the library's own tensor tables) and its tasks."""
    sh = setup.shape
    mbt = max_batch_tokens or max(256, int(sh.batch_tokens * 1.5))
    ctx = Context(sh.d_model, sh.n_heads, sh.d_ff, sh.vocab, sh.dtype, sh.max_len, min(16384, mbt),
                  sh.label_smoothing, sh.adam_beta1, sh.adam_beta2, sh.adam_eps, sh.ln_eps,
                  hip_stream=hip_stream, plan_only=plan_only)
    for k, ms in enumerate(setup.modules):
        j = ctx.mm_register_module(ms.kind, ms.name, ms.position, ms.n_layers, ms.owns_final_norm,
                                   ms.adapter_dim, ms.stack)
        if fill_params is not None and not plan_only:
            table, total = ctx.mm_get_layout(j)
            init = fill_params([(role, off, rows * cols) for role, off, rows, cols in table], total,
                               setup.weight_seed * 1000 + k, perturbed)
            ctx.mm_set_params(j, init)
    for _, ids in setup.tasks:
        ctx.mm_route_task(ids)
    return ctx
