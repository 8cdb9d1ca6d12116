"""ctypes binding of the CPU oracle (test infrastructure only: tests, smoke, bench cpu_baseline).

Marshals numpy arrays into ``libee_oracle.so``; holds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

EO_F32, EO_BF16 = 0, 1


class EoConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("n_exits", C.c_int32), ("exit_layers", C.c_int32 * 8), ("dtype", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("exit_flags", C.c_int32)]


EO_EXIT_NO_NORM, EO_TIE_EMBEDDINGS, EO_EXIT_MLP, EO_EXIT_LAYER = 1, 2, 4, 8


class EoDiag(C.Structure):
    _fields_ = [("layer", C.c_int32), ("argmax", C.c_int32), ("arg2", C.c_int32), ("conf", C.c_float),
                ("top1", C.c_float), ("top2", C.c_float)]

    def as_dict(self):
        return dict(layer=self.layer, argmax=self.argmax, arg2=self.arg2, conf=self.conf,
                    top1=self.top1, top2=self.top2)


_lib = None


def lib():
    global _lib
    if _lib is None:
        # EE_ORACLE_LIB: another build of the same source (the sanitizer build of oracle/build.py)
        path = os.environ.get("EE_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        vp, i32p, fp = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
        L.eo_model_create.restype = vp
        L.eo_model_create.argtypes = [C.POINTER(EoConfig)]
        L.eo_model_set_tensor.argtypes = [vp, C.c_int, C.c_int, vp]
        L.eo_model_free.argtypes = [vp]
        L.eo_generate_g0.argtypes = [vp, i32p, C.c_int, C.c_int, C.c_float, i32p, i32p]
        L.eo_generate_g0_capped.argtypes = [vp, i32p, C.c_int, C.c_int, C.c_float, C.c_int, i32p, i32p]
        L.eo_generate_plain.argtypes = [vp, i32p, C.c_int, C.c_int, i32p]
        L.eo_forward_sequence.argtypes = [vp, i32p, C.c_int, fp, fp, fp]
        L.eo_exit_layer_sequence.argtypes = [vp, C.c_int, fp, C.c_int, fp, fp, fp]
        L.eo_state_create.restype = vp
        L.eo_state_create.argtypes = [vp, C.c_int, C.c_int]
        L.eo_state_free.argtypes = [vp]
        L.eo_prefill.argtypes = [vp, i32p, C.c_int, C.POINTER(EoDiag)]
        L.eo_step_begin.argtypes = [vp, C.c_int32]
        L.eo_step_advance.argtypes = [vp, C.c_int, C.POINTER(EoDiag)]
        L.eo_step_commit.argtypes = [vp, C.c_int32]
        L.eo_decode_step.argtypes = [vp, C.c_int32, C.c_float, i32p, i32p, fp]
        L.eo_flush.argtypes = [vp]
        L.eo_filled.argtypes = [vp, C.c_int]
        L.eo_n_pending.argtypes = [vp]
        L.eo_kv_read.argtypes = [vp, C.c_int, C.c_int, C.c_int, fp, fp]
        L.eo_last_hidden.argtypes = [vp, fp]
        L.eo_last_logits.argtypes = [vp, fp]
        L.eo_bf16_round.restype = C.c_float
        L.eo_bf16_round.argtypes = [C.c_float]
        L.eo_norm_matvec.restype = None
        L.eo_norm_matvec.argtypes = [C.c_int, vp, C.c_int, C.c_int, fp, fp, C.c_float, fp]
        L.eo_rope.restype = None
        L.eo_rope.argtypes = [fp, C.c_int, C.c_int, C.c_int, C.c_float]
        L.eo_attention_row.restype = None
        L.eo_attention_row.argtypes = [fp, fp, fp, C.c_int, C.c_int, C.c_int, fp]
        L.eo_swiglu.restype = None
        L.eo_swiglu.argtypes = [fp, fp, C.c_int, fp]
        L.eo_softmax_max.restype = None
        L.eo_softmax_max.argtypes = [fp, C.c_int, C.POINTER(EoDiag)]
        L.eo_layer_row.argtypes = [vp, C.c_int, fp, C.c_int, fp, fp]
        L.eo_head_row.argtypes = [vp, C.c_int, fp, fp, C.POINTER(EoDiag)]
        L.eo_set_threads.restype = None
        L.eo_set_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _fp(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _ip(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def set_threads(n: int) -> None:
    lib().eo_set_threads(int(n))


def get_threads() -> int:
    return int(lib().eo_get_threads())


def make_config(n_layers, d_model, n_heads, head_dim, d_ff, vocab, exit_layers, dtype,
                rms_eps=1e-5, rope_base=10000.0, exit_flags=0) -> EoConfig:
    c = EoConfig()
    c.n_layers, c.d_model, c.n_heads, c.head_dim, c.d_ff, c.vocab = n_layers, d_model, n_heads, head_dim, d_ff, vocab
    c.n_exits = len(exit_layers)
    for i, e in enumerate(exit_layers):
        c.exit_layers[i] = e
    c.dtype = EO_BF16 if dtype in ("bf16", EO_BF16) else EO_F32
    c.rms_eps, c.rope_base = rms_eps, rope_base
    c.exit_flags = exit_flags
    return c


class Model:
    """An oracle model over borrowed numpy arrays (float32, or uint16 holding bf16 bit patterns)."""

    def __init__(self, cfg: EoConfig):
        self.cfg = cfg
        self.h = lib().eo_model_create(C.byref(cfg))
        if not self.h:
            raise ValueError("oracle: bad config")
        self._keep: Dict[Tuple[int, int], np.ndarray] = {}

    def set_tensor(self, kind: int, index: int, arr: np.ndarray) -> None:
        arr = np.ascontiguousarray(arr)
        self._keep[(int(kind), int(index))] = arr
        if lib().eo_model_set_tensor(self.h, int(kind), int(index), arr.ctypes.data):
            raise ValueError(f"oracle: bad tensor {kind} {index}")

    def tensor(self, kind: int, index: int) -> np.ndarray:
        return self._keep[(int(kind), int(index))]

    def close(self):
        if self.h and _lib is not None:
            _lib.eo_model_free(self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- G0 and friends
    def generate_g0(self, prompt: Sequence[int], n_new: int, threshold: float, max_pending: int = 0):
        p = np.asarray(prompt, dtype=np.int32)
        toks = np.zeros(n_new, np.int32)
        ex = np.zeros(n_new, np.int32)
        rc = lib().eo_generate_g0_capped(self.h, _ip(p), len(p), n_new, threshold, max_pending, _ip(toks), _ip(ex))
        if rc:
            raise RuntimeError("eo_generate_g0 failed")
        return toks, ex

    def generate_plain(self, prompt: Sequence[int], n_new: int):
        p = np.asarray(prompt, dtype=np.int32)
        toks = np.zeros(n_new, np.int32)
        if lib().eo_generate_plain(self.h, _ip(p), len(p), n_new, _ip(toks)):
            raise RuntimeError("eo_generate_plain failed")
        return toks

    def forward_sequence(self, tokens: Sequence[int]):
        t = np.asarray(tokens, dtype=np.int32)
        n, d, L = len(t), self.cfg.d_model, self.cfg.n_layers
        hid = np.zeros((L + 1, n, d), np.float32)
        k = np.zeros((L, n, d), np.float32)
        v = np.zeros((L, n, d), np.float32)
        if lib().eo_forward_sequence(self.h, _ip(t), n, _fp(hid), _fp(k), _fp(v)):
            raise RuntimeError("eo_forward_sequence failed")
        return hid, k, v

    def exit_layer_sequence(self, exit_index: int, hidden: np.ndarray):
        """The exit's own Transformer layer over hidden states [n][d] -> (x_out, k, v), each [n][d]."""
        hidden = np.ascontiguousarray(hidden, dtype=np.float32)
        n, d = hidden.shape
        x, k, v = (np.zeros((n, d), np.float32) for _ in range(3))
        if lib().eo_exit_layer_sequence(self.h, exit_index, _fp(hidden), n, _fp(x), _fp(k), _fp(v)):
            raise RuntimeError("eo_exit_layer_sequence failed")
        return x, k, v

    def layer_row(self, layer: int, x: np.ndarray, pos: int, K: np.ndarray, V: np.ndarray) -> None:
        if lib().eo_layer_row(self.h, layer, _fp(x), pos, _fp(K), _fp(V)):
            raise RuntimeError("eo_layer_row failed")

    def head_row(self, head: int, x: np.ndarray):
        z = np.zeros(self.cfg.vocab, np.float32)
        d = EoDiag()
        if lib().eo_head_row(self.h, head, _fp(x), _fp(z), C.byref(d)):
            raise RuntimeError("eo_head_row failed")
        return z, d.as_dict()


class State:
    """G1: KV cache + pending list + recomputation, one sequence."""

    def __init__(self, model: Model, max_positions: int, max_pending: int):
        self.model = model
        self.h = lib().eo_state_create(model.h, max_positions, max_pending)
        if not self.h:
            raise ValueError("oracle: bad state")

    def close(self):
        if self.h and _lib is not None:
            _lib.eo_state_free(self.h)
        self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens: Sequence[int]) -> List[dict]:
        t = np.asarray(tokens, dtype=np.int32)
        n = self.model.cfg.n_exits + 1
        dg = (EoDiag * n)()
        if lib().eo_prefill(self.h, _ip(t), len(t), dg):
            raise RuntimeError("eo_prefill failed")
        return [dg[i].as_dict() for i in range(n)]

    def step_begin(self, token: int) -> bool:
        rc = lib().eo_step_begin(self.h, int(token))
        if rc < 0:
            raise RuntimeError("eo_step_begin failed")
        return bool(rc)

    def step_advance(self, eval_head: bool) -> Tuple[int, Optional[dict]]:
        d = EoDiag()
        d.layer = -1
        depth = lib().eo_step_advance(self.h, int(eval_head), C.byref(d))
        if depth < 0:
            raise RuntimeError("eo_step_advance failed")
        return depth, (d.as_dict() if d.layer >= 0 else None)

    def step_commit(self, token: int) -> None:
        if lib().eo_step_commit(self.h, int(token)):
            raise RuntimeError("eo_step_commit failed")

    def decode_step(self, token: int, threshold: float) -> Tuple[int, int, float]:
        nt, ex, cf = C.c_int32(), C.c_int32(), C.c_float()
        if lib().eo_decode_step(self.h, int(token), threshold, C.byref(nt), C.byref(ex), C.byref(cf)):
            raise RuntimeError("eo_decode_step failed")
        return nt.value, ex.value, cf.value

    def flush(self) -> None:
        if lib().eo_flush(self.h):
            raise RuntimeError("eo_flush failed")

    def filled(self, segment: int) -> int:
        return int(lib().eo_filled(self.h, segment))

    def n_pending(self) -> int:
        return int(lib().eo_n_pending(self.h))

    def kv_read(self, layer: int, pos0: int, n: int):
        d = self.model.cfg.d_model
        k = np.zeros((n, d), np.float32)
        v = np.zeros((n, d), np.float32)
        if lib().eo_kv_read(self.h, layer, pos0, n, _fp(k), _fp(v)):
            raise RuntimeError("eo_kv_read failed")
        return k, v

    def last_hidden(self) -> np.ndarray:
        x = np.zeros(self.model.cfg.d_model, np.float32)
        lib().eo_last_hidden(self.h, _fp(x))
        return x

    def last_logits(self) -> np.ndarray:
        z = np.zeros(self.model.cfg.vocab, np.float32)
        lib().eo_last_logits(self.h, _fp(z))
        return z


# ---- single operations (for pins)

def bf16_round(v: float) -> float:
    return float(lib().eo_bf16_round(v))


def norm_matvec(dtype: int, W: np.ndarray, x: np.ndarray, g: Optional[np.ndarray], eps: float) -> np.ndarray:
    N, K = W.shape
    y = np.zeros(N, np.float32)
    W = np.ascontiguousarray(W)
    lib().eo_norm_matvec(dtype, W.ctypes.data, N, K, _fp(x), _fp(g) if g is not None else None, eps, _fp(y))
    return y


def rope(vec: np.ndarray, n_heads: int, head_dim: int, pos: int, base: float) -> np.ndarray:
    out = np.ascontiguousarray(vec, dtype=np.float32).copy()
    lib().eo_rope(_fp(out), n_heads, head_dim, pos, base)
    return out


def attention_row(q: np.ndarray, K: np.ndarray, V: np.ndarray, n_heads: int, head_dim: int):
    out = np.zeros(n_heads * head_dim, np.float32)
    lib().eo_attention_row(_fp(q), _fp(K), _fp(V), K.shape[0], n_heads, head_dim, _fp(out))
    return out


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    out = np.zeros_like(gate)
    lib().eo_swiglu(_fp(gate), _fp(up), len(gate), _fp(out))
    return out


def softmax_max(z: np.ndarray) -> dict:
    d = EoDiag()
    lib().eo_softmax_max(_fp(z), len(z), C.byref(d))
    return d.as_dict()
