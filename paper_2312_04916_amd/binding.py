"""ctypes binding of include/ee.h (argument marshalling only) plus small RAII helpers that own the
torch device buffers the library works in."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

EE_F32, EE_BF16 = 0, 1
EE_MAX_ROWS, EE_MAX_SEQS, EE_MAX_EXITS = 256, 64, 8
EE_K_QKV, EE_K_ATTN, EE_K_OPROJ, EE_K_SWIGLU, EE_K_DOWN, EE_K_HEAD = range(6)
KERNEL_NAMES = ["qkv", "attention", "oproj", "swiglu", "down", "head"]
(EE_T_EMBED, EE_T_ATTN_NORM, EE_T_WQ, EE_T_WK, EE_T_WV, EE_T_WO, EE_T_MLP_NORM, EE_T_WG, EE_T_WU, EE_T_WD,
 EE_T_EXIT_NORM, EE_T_EXIT_HEAD, EE_T_FINAL_NORM, EE_T_FINAL_HEAD) = range(14)

EXPORTS = ["ee_strerror", "ee_last_hip_error", "ee_model_bytes", "ee_model_create", "ee_model_set_tensor",
           "ee_model_load", "ee_model_free", "ee_debug_set_logits", "ee_debug_step_confidences", "ee_debug_plan", "ee_profile_begin", "ee_profile_end", "ee_profile_every", "ee_measure_stream_read", "ee_debug_lane_reductions", "ee_kv_cache_bytes", "ee_kv_cache_create",
           "ee_kv_cache_set_refeed", "ee_kv_cache_set_pipeline", "ee_kv_cache_reset", "ee_kv_cache_filled", "ee_kv_cache_pending", "ee_kv_cache_read",
           "ee_kv_cache_flush", "ee_kv_cache_free", "ee_debug_read_hidden", "ee_prefill", "ee_prefill_scored",
           "ee_decode_step", "ee_decode_step_static"]

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libee.so")


class ee_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("n_exits", C.c_int32),
                ("exit_layers", C.c_int32 * EE_MAX_EXITS), ("dtype", C.c_int32), ("max_positions", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("exit_flags", C.c_int32),
                ("prefill_rows", C.c_int32), ("gemm_min_workgroups", C.c_int32), ("scored_head_terms", C.c_int32)]


EE_EXIT_NO_NORM, EE_TIE_EMBEDDINGS, EE_EXIT_MLP, EE_EXIT_LAYER = 1, 2, 4, 8
(EE_T_EXIT_MLP_NORM, EE_T_EXIT_WG, EE_T_EXIT_WU, EE_T_EXIT_WD, EE_T_EXIT_ATTN_NORM, EE_T_EXIT_WQ, EE_T_EXIT_WK, EE_T_EXIT_WV,
 EE_T_EXIT_WO) = range(14, 23)


class EeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().ee_strerror(code).decode()
        if code == -6:
            msg += f" (hip status {lib().ee_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


_lib = None


def lib():
    """Loads libee.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_04916_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32p, fp = C.c_void_p, C.c_size_t, C.POINTER(C.c_int32), C.POINTER(C.c_float)
        L.ee_strerror.restype = C.c_char_p
        L.ee_strerror.argtypes = [C.c_int]
        L.ee_last_hip_error.argtypes = []
        L.ee_model_bytes.argtypes = [C.POINTER(ee_config), C.c_int, C.c_int, C.POINTER(sz), C.POINTER(sz)]
        L.ee_model_create.argtypes = [C.POINTER(ee_config), vp, sz, vp, sz, C.c_int, C.c_int, vp, C.POINTER(vp)]
        L.ee_model_set_tensor.argtypes = [vp, C.c_int, C.c_int, vp, sz, vp]
        L.ee_model_load.argtypes = [C.POINTER(ee_config), C.c_char_p, vp, sz, vp, sz, C.c_int, C.c_int, vp, sz, vp,
                                    C.POINTER(vp)]
        L.ee_model_free.argtypes = [vp]
        L.ee_debug_set_logits.argtypes = [vp, vp, C.c_int]
        L.ee_debug_step_confidences.argtypes = [vp, C.c_int, fp]
        L.ee_debug_plan.argtypes = [C.c_int, i32p, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p]
        L.ee_profile_begin.argtypes = [vp, C.c_int, C.c_int]
        L.ee_profile_end.argtypes = [vp, i32p, fp]
        L.ee_profile_every.argtypes = [vp, C.c_int]
        L.ee_measure_stream_read.argtypes = [vp, sz, C.c_int, fp, vp]
        L.ee_debug_lane_reductions.argtypes = [vp, i32p, vp]
        L.ee_kv_cache_bytes.argtypes = [vp, C.c_int, C.c_int64, C.c_int, C.c_int, C.POINTER(sz)]
        L.ee_kv_cache_create.argtypes = [vp, C.c_int, C.c_int64, C.c_int, C.c_int, vp, sz, C.POINTER(vp)]
        L.ee_kv_cache_reset.argtypes = [vp, C.c_int]
        L.ee_kv_cache_set_refeed.argtypes = [vp, C.c_int]
        L.ee_kv_cache_set_pipeline.argtypes = [vp, vp, vp, sz, vp]
        L.ee_kv_cache_filled.argtypes = [vp, C.c_int, C.c_int, i32p]
        L.ee_kv_cache_pending.argtypes = [vp, C.c_int, i32p]
        L.ee_kv_cache_read.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, fp, fp, vp]
        L.ee_kv_cache_flush.argtypes = [vp, vp, C.c_int, i32p, vp]
        L.ee_kv_cache_free.argtypes = [vp]
        L.ee_debug_read_hidden.argtypes = [vp, vp, C.c_int, fp, vp]
        L.ee_prefill.argtypes = [vp, vp, C.c_int, i32p, C.c_int, C.c_float, i32p, i32p, fp, vp]
        L.ee_prefill_scored.argtypes = [vp, vp, C.c_int, i32p, C.c_int, C.c_float, i32p, i32p, fp, i32p, fp, fp, vp]
        # (the step's arrays go in as plain addresses: building a typed ctypes pointer per array and call cost the
        # step 40 us of host time)
        L.ee_decode_step.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp, C.c_float, vp, vp, vp, vp]
        L.ee_decode_step_static.argtypes = L.ee_decode_step.argtypes
        _lib = L
    return _lib


def _chk(code: int, where: str) -> None:
    if code != 0:
        raise EeError(code, where)


def make_config(n_layers, d_model, n_heads, head_dim, d_ff, vocab, exit_layers, dtype, max_positions,
                rms_eps=1e-5, rope_base=10000.0, exit_flags=0, prefill_rows=0, gemm_min_workgroups=0,
                scored_head_terms=0) -> ee_config:
    c = ee_config()
    c.n_layers, c.d_model, c.n_heads, c.head_dim, c.d_ff, c.vocab = n_layers, d_model, n_heads, head_dim, d_ff, vocab
    c.n_exits = len(exit_layers)
    for i, e in enumerate(exit_layers):
        c.exit_layers[i] = e
    c.dtype = EE_BF16 if dtype in ("bf16", EE_BF16) else EE_F32
    c.max_positions = max_positions
    c.rms_eps, c.rope_base = rms_eps, rope_base
    c.exit_flags = exit_flags
    c.prefill_rows, c.gemm_min_workgroups, c.scored_head_terms = prefill_rows, gemm_min_workgroups, scored_head_terms
    return c


def config_of_shape(shape, max_positions: int, prefill_rows: int = 0, gemm_min_workgroups: int = 0,
                    scored_head_terms: int = 0) -> ee_config:
    """ee_config of an object with the model-shape fields (n_layers, d_model, n_heads, head_dim, d_ff, vocab,
    exit_layers, dtype, rms_eps, rope_base, exit_flags), e.g. workload.ModelShape."""
    return make_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff, shape.vocab,
                       shape.exit_layers, shape.dtype, max_positions, shape.rms_eps, shape.rope_base, shape.exit_flags,
                       prefill_rows, gemm_min_workgroups, scored_head_terms)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


class Model:
    """Owns the weight and workspace buffers (torch, device) and the ee_model handle."""

    def __init__(self, cfg: ee_config, max_rows: int = 64, max_seqs: int = 1, device="cuda:0", stream=None):
        self.cfg, self.max_rows, self.max_seqs = cfg, max_rows, max_seqs
        self.device = torch.device(device)
        wb, sb = C.c_size_t(), C.c_size_t()
        _chk(lib().ee_model_bytes(C.byref(cfg), max_rows, max_seqs, C.byref(wb), C.byref(sb)), "ee_model_bytes")
        self.weight_bytes, self.workspace_bytes = wb.value, sb.value
        self.weights = torch.empty(wb.value, dtype=torch.uint8, device=self.device)
        self.workspace = torch.zeros(sb.value, dtype=torch.uint8, device=self.device)
        self.h = C.c_void_p()
        _chk(lib().ee_model_create(C.byref(cfg), self.weights.data_ptr(), wb.value, self.workspace.data_ptr(), sb.value,
                                   max_rows, max_seqs, _stream_ptr(stream), C.byref(self.h)), "ee_model_create")
        self._logits = None

    def set_tensor(self, kind: int, index: int, t: torch.Tensor, stream=None) -> None:
        assert t.is_cuda and t.is_contiguous()
        _chk(lib().ee_model_set_tensor(self.h, kind, index, t.data_ptr(), t.numel(), _stream_ptr(stream)),
             f"ee_model_set_tensor({kind},{index})")

    def enable_logits(self, rows: int = 1) -> torch.Tensor:
        self._logits = torch.zeros(rows, self.cfg.vocab, dtype=torch.float32, device=self.device)
        _chk(lib().ee_debug_set_logits(self.h, self._logits.data_ptr(), rows), "ee_debug_set_logits")
        return self._logits

    def step_confidences(self, n_seqs: int = 1) -> np.ndarray:
        """ee_debug_step_confidences -> float32[n_seqs][n_exits+1], -1 where a head was not evaluated in the last step."""
        out = np.zeros((n_seqs, self.cfg.n_exits + 1), np.float32)
        _chk(lib().ee_debug_step_confidences(self.h, n_seqs, _fp(out)), "ee_debug_step_confidences")
        return out

    def profile_begin(self, kernel: int, max_launches: int = 16384, every: int = 1) -> None:
        _chk(lib().ee_profile_every(self.h, every), "ee_profile_every")
        _chk(lib().ee_profile_begin(self.h, kernel, max_launches), "ee_profile_begin")

    def profile_end(self) -> Tuple[int, float]:
        n, ms = C.c_int32(), C.c_float()
        _chk(lib().ee_profile_end(self.h, C.byref(n), C.byref(ms)), "ee_profile_end")
        return n.value, ms.value

    def measure_stream_read(self, n_bytes: int = 0, n_launches: int = 20) -> float:
        """GB/s (1e9) of a read-only kernel over n_bytes of the weight buffer (0: all of it)."""
        g = C.c_float()
        _chk(lib().ee_measure_stream_read(self.h, n_bytes, n_launches, C.byref(g), _stream_ptr(None)), "ee_measure_stream_read")
        return g.value

    def lane_reduction_mismatches(self) -> int:
        """ee_debug_lane_reductions: results of the kernels' lane reductions that differ from the shuffle butterflies."""
        n = C.c_int32(-1)
        _chk(lib().ee_debug_lane_reductions(self.h, C.byref(n), _stream_ptr(None)), "ee_debug_lane_reductions")
        return n.value

    def close(self):
        if self.h:
            torch.cuda.synchronize()
            lib().ee_model_free(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def model_load(cfg: ee_config, path: str, max_rows: int = 64, max_seqs: int = 1, device="cuda:0", stream=None) -> Model:
    """ee_model_load: a Model whose tensors come from a weight file."""
    m = Model.__new__(Model)
    m.cfg, m.max_rows, m.max_seqs, m.device, m._logits = cfg, max_rows, max_seqs, torch.device(device), None
    wb, sb = C.c_size_t(), C.c_size_t()
    _chk(lib().ee_model_bytes(C.byref(cfg), max_rows, max_seqs, C.byref(wb), C.byref(sb)), "ee_model_bytes")
    m.weight_bytes, m.workspace_bytes = wb.value, sb.value
    m.weights = torch.empty(wb.value, dtype=torch.uint8, device=m.device)
    m.workspace = torch.zeros(sb.value, dtype=torch.uint8, device=m.device)
    es = 2 if cfg.dtype == EE_BF16 else 4
    staging_bytes = max(cfg.vocab, cfg.d_ff, cfg.d_model) * cfg.d_model * es
    staging = torch.empty(staging_bytes, dtype=torch.uint8, device=m.device)
    m.h = C.c_void_p()
    _chk(lib().ee_model_load(C.byref(cfg), path.encode(), m.weights.data_ptr(), wb.value, m.workspace.data_ptr(), sb.value,
                             max_rows, max_seqs, staging.data_ptr(), staging_bytes, _stream_ptr(stream), C.byref(m.h)),
         "ee_model_load")
    torch.cuda.synchronize()
    return m


class KvCache:
    """Owns the cache pool (torch, device) and the ee_kv_cache handle."""

    def __init__(self, model: Model, max_seqs: int, max_tokens_total: int, block_tokens: int = 64, max_pending: int = 15):
        self.model = model
        nb = C.c_size_t()
        _chk(lib().ee_kv_cache_bytes(model.h, max_seqs, max_tokens_total, block_tokens, max_pending, C.byref(nb)),
             "ee_kv_cache_bytes")
        self.pool_bytes = nb.value
        self.pool = torch.zeros(nb.value, dtype=torch.uint8, device=model.device)
        self.h = C.c_void_p()
        _chk(lib().ee_kv_cache_create(model.h, max_seqs, max_tokens_total, block_tokens, max_pending, self.pool.data_ptr(),
                                      nb.value, C.byref(self.h)), "ee_kv_cache_create")

    def reset(self, seq: int) -> None:
        _chk(lib().ee_kv_cache_reset(self.h, seq), "ee_kv_cache_reset")

    def set_refeed(self, on: bool) -> None:
        _chk(lib().ee_kv_cache_set_refeed(self.h, 1 if on else 0), "ee_kv_cache_set_refeed")

    def set_pipeline(self, on: bool = True) -> None:
        """ee_kv_cache_set_pipeline: pipeline-based early exit, with a second workspace and a second stream (both owned
        here); on=False returns to KV recomputation."""
        if not on:
            _chk(lib().ee_kv_cache_set_pipeline(self.model.h, self.h, None, 0, None), "ee_kv_cache_set_pipeline")
            self._fill_ws = self._fill_stream = None
            return
        self._fill_ws = torch.zeros(self.model.workspace_bytes, dtype=torch.uint8, device=self.model.device)
        self._fill_stream = torch.cuda.Stream(device=self.model.device)
        torch.cuda.synchronize()
        _chk(lib().ee_kv_cache_set_pipeline(self.model.h, self.h, self._fill_ws.data_ptr(), self.model.workspace_bytes,
                                            C.c_void_p(self._fill_stream.cuda_stream)), "ee_kv_cache_set_pipeline")

    def filled(self, seq: int, layer: int) -> int:
        n = C.c_int32()
        _chk(lib().ee_kv_cache_filled(self.h, seq, layer, C.byref(n)), "ee_kv_cache_filled")
        return n.value

    def pending(self, seq: int) -> int:
        n = C.c_int32()
        _chk(lib().ee_kv_cache_pending(self.h, seq, C.byref(n)), "ee_kv_cache_pending")
        return n.value

    def read(self, seq: int, layer: int, pos0: int, n: int, stream=None) -> Tuple[np.ndarray, np.ndarray]:
        d = self.model.cfg.d_model
        k = np.zeros((n, d), np.float32)
        v = np.zeros((n, d), np.float32)
        _chk(lib().ee_kv_cache_read(self.model.h, self.h, seq, layer, pos0, n, _fp(k), _fp(v), _stream_ptr(stream)),
             "ee_kv_cache_read")
        return k, v

    def flush(self, seq_ids: Sequence[int], stream=None) -> None:
        s = _i32(seq_ids)
        _chk(lib().ee_kv_cache_flush(self.model.h, self.h, len(s), _ip(s), _stream_ptr(stream)), "ee_kv_cache_flush")

    def read_hidden(self, seq: int, stream=None) -> np.ndarray:
        x = np.zeros(self.model.cfg.d_model, np.float32)
        _chk(lib().ee_debug_read_hidden(self.model.h, self.h, seq, _fp(x), _stream_ptr(stream)), "ee_debug_read_hidden")
        return x

    def close(self):
        if self.h:
            torch.cuda.synchronize()
            lib().ee_kv_cache_free(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan(filled: Sequence[int], position: int, max_pending: int, refeed: bool = False, reached: int = -1):
    """ee_debug_plan (host only) -> (forced, [(lo, hi) per segment], watermarks after the optional commit)."""
    n = len(filled)
    f = (C.c_int32 * n)(*[int(v) for v in filled])
    lo, hi = (C.c_int32 * n)(), (C.c_int32 * n)()
    forced = C.c_int32()
    _chk(lib().ee_debug_plan(n, f, int(position), int(max_pending), int(bool(refeed)), int(reached), C.byref(forced), lo, hi),
         "ee_debug_plan")
    return bool(forced.value), [(lo[i], hi[i]) for i in range(n)], [f[i] for i in range(n)]


def prefill(model: Model, cache: KvCache, seq: int, tokens: Sequence[int], threshold: float, stream=None):
    """ee_prefill -> (next_token, exit_layer, conf[n_exits+1])."""
    t = _i32(tokens)
    nt, ex = C.c_int32(), C.c_int32()
    conf = np.zeros(model.cfg.n_exits + 1, np.float32)
    _chk(lib().ee_prefill(model.h, cache.h, seq, _ip(t), len(t), threshold, C.byref(nt), C.byref(ex), _fp(conf),
                          _stream_ptr(stream)), "ee_prefill")
    return nt.value, ex.value, conf


def prefill_scored(model: Model, cache: KvCache, seq: int, tokens: Sequence[int], threshold: float, stream=None, nll: bool = False):
    """ee_prefill_scored -> (next_token, exit_layer, conf[n_exits+1], pos_token[n_exits+1][n], pos_conf[n_exits+1][n])
    and, with nll=True, pos_nll[n_exits+1][n] as a sixth element."""
    t = _i32(tokens)
    nt, ex = C.c_int32(), C.c_int32()
    nh = model.cfg.n_exits + 1
    conf = np.zeros(nh, np.float32)
    ptok = np.zeros((nh, len(t)), np.int32)
    pconf = np.zeros((nh, len(t)), np.float32)
    pnll = np.zeros((nh, len(t)), np.float32) if nll else None
    _chk(lib().ee_prefill_scored(model.h, cache.h, seq, _ip(t), len(t), threshold, C.byref(nt), C.byref(ex), _fp(conf),
                                 _ip(ptok), _fp(pconf), _fp(pnll) if nll else None, _stream_ptr(stream)), "ee_prefill_scored")
    if nll:
        return nt.value, ex.value, conf, ptok, pconf, pnll
    return nt.value, ex.value, conf, ptok, pconf


def decode_step(model: Model, cache: KvCache, seq_ids: Sequence[int], row_offsets: Sequence[int], tokens: Sequence[int],
                pending_mask: Sequence[int], threshold: float, stream=None, static_workspace: bool = False):
    """ee_decode_step (or ee_decode_step_static) -> (next_token[n], exit_layer[n], conf[n])."""
    s, ro, tk = _i32(seq_ids), _i32(row_offsets), _i32(tokens)
    pm = np.ascontiguousarray(np.asarray(pending_mask, dtype=np.uint8))
    n = len(s)
    nt, ex, cf = np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.float32)
    fn = lib().ee_decode_step_static if static_workspace else lib().ee_decode_step
    code = fn(model.h, cache.h, n, s.ctypes.data, ro.ctypes.data, tk.ctypes.data, pm.ctypes.data, threshold, nt.ctypes.data,
              ex.ctypes.data, cf.ctypes.data, _stream_ptr(stream))
    if code != 0:
        _chk(code, "ee_decode_step")
    return nt, ex, cf


class Sequences:
    """Caller-side bookkeeping of the deferred-token lists that ee_decode_step expects: every token
    emitted since the last step that ran to full depth, oldest first, then the current token."""

    def __init__(self, n_layers: int, pipeline: bool = False):
        self.n_layers = n_layers
        self.pipeline = pipeline  # pipeline-based early exit: the library defers nothing, the lists stay empty
        self.pending: dict = {}
        self.current: dict = {}

    def start(self, seq: int, first_token: int) -> None:
        self.pending[seq] = []
        self.current[seq] = int(first_token)

    def rows(self, seq_ids: Sequence[int]):
        ro, tk, pm = [0], [], []
        for s in seq_ids:
            tk += self.pending[s] + [self.current[s]]
            pm += [1] * len(self.pending[s]) + [0]
            ro.append(len(tk))
        return ro, tk, pm

    def update(self, seq_ids: Sequence[int], next_token, exit_layer) -> None:
        for i, s in enumerate(seq_ids):
            if int(exit_layer[i]) == self.n_layers or self.pipeline:
                self.pending[s] = []
            else:
                self.pending[s].append(self.current[s])
            self.current[s] = int(next_token[i])
