"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and the
host-side argument validation that needs no GPU returns the documented error codes."""
import ctypes as C
import os
import re

import pytest

import paper_2312_04916_amd as ee
from workload import CONFIGS

from common import ee_config_of

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ee.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ee_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ee.lib()
    names = declared_symbols()
    assert len(names) >= 19
    for n in names:
        assert hasattr(L, n), f"{n} is declared in ee.h but not exported"
    assert sorted(ee.EXPORTS) == names


def test_strerror_names_every_code():
    L = ee.lib()
    seen = {L.ee_strerror(c).decode() for c in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown error" not in seen
    assert L.ee_strerror(-99).decode() == "unknown error"


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C5"])
def test_model_bytes_accounts_for_every_parameter(name):
    w = CONFIGS[name]
    cfg = ee_config_of(w.shape, 4096)
    wb, sb = C.c_size_t(), C.c_size_t()
    assert ee.lib().ee_model_bytes(C.byref(cfg), 64, 4, C.byref(wb), C.byref(sb)) == 0
    es = 2 if w.shape.dtype == "bf16" else 4
    n_gain = (2 * w.shape.n_layers + len(w.shape.exit_layers) + 1) * w.shape.d_model
    lower = (w.shape.n_params() - n_gain) * es + n_gain * 4
    assert lower <= wb.value <= lower * 1.01 + (1 << 22)
    assert sb.value > 0


def test_bad_configs_are_rejected():
    L = ee.lib()
    wb = C.c_size_t()
    good = CONFIGS["C1"].shape

    def code(**kw):
        cfg = ee_config_of(good, 256)
        for k, v in kw.items():
            setattr(cfg, k, v)
        return L.ee_model_bytes(C.byref(cfg), 16, 1, C.byref(wb), None)

    assert code() == 0
    assert code(head_dim=48) == -1          # unsupported head size
    assert code(n_heads=3) == -1            # d_model != n_heads*head_dim
    assert code(d_ff=100) == -1             # not a multiple of 32
    assert code(dtype=7) == -1
    assert code(max_positions=0) == -1
    assert code(scored_head_terms=2) == 0 and code(scored_head_terms=3) == -1 and code(scored_head_terms=-1) == -1
    cfg = ee_config_of(good, 256)
    cfg.exit_layers[0], cfg.exit_layers[1] = 2, 1  # not ascending
    assert L.ee_model_bytes(C.byref(cfg), 16, 1, C.byref(wb), None) == -1
    cfg = ee_config_of(good, 256)
    cfg.exit_layers[1] = 4                  # an exit after the last layer is the final head
    assert L.ee_model_bytes(C.byref(cfg), 16, 1, C.byref(wb), None) == -1
    cfg = ee_config_of(good, 256)
    assert L.ee_model_bytes(C.byref(cfg), 0, 1, C.byref(wb), None) == -1
    assert L.ee_model_bytes(C.byref(cfg), 16, 65, C.byref(wb), None) == -1
    assert L.ee_model_bytes(None, 16, 1, C.byref(wb), None) == -7


# ---------------------------------------------------------------- the step plan (host logic, no GPU)

def _oracle_run(tau, cap, n_new=40):
    """Drives the oracle's KV-recomputation generator and yields, per decode step, its state before the step
    (watermarks, deferred count), whether the step was forced, and the segment it ended in."""
    from oracle import oracle as O
    from oracle.from_workload import build_model
    from workload import prompt_tokens

    shape = CONFIGS["C1"].shape
    om = build_model(shape, 0, gain_jitter=0.1)
    p = prompt_tokens(shape.vocab, 16, 1).numpy()
    st = O.State(om, 16 + n_new + 1, cap)
    diags = st.prefill(p)
    tok = diags[-1]["argmax"]
    if tau < 1.0:
        for dg in diags[:-1]:
            if dg["conf"] >= tau:
                tok = dg["argmax"]
                break
    n_seg = len(shape.exit_layers) + 1
    seg_of = {e: i for i, e in enumerate(list(shape.exit_layers) + [shape.n_layers])}
    pos = 16
    for _ in range(n_new):
        before = [st.filled(s) for s in range(n_seg)]
        pend = st.n_pending()
        forced = st.step_begin(tok)
        evaluated = (not forced) and tau < 1.0
        while True:
            depth, dg = st.step_advance(evaluated)
            if depth == shape.n_layers or (dg is not None and dg["conf"] >= tau):
                break
        st.step_commit(dg["argmax"])
        tok = dg["argmax"]
        yield before, pend, pos, forced, seg_of[depth], [st.filled(s) for s in range(n_seg)]
        pos += 1


@pytest.mark.parametrize("tau,cap", [(0.0, 3), (0.0, 15), (0.2, 6), (0.35, 40), (0.5, 2), (1.0, 5), (0.0, 0), (0.2, -1)])
def test_step_plan_follows_the_oracle_state(tau, cap):
    """The library's host-side plan (forced full pass at the cap, rows per segment, watermark updates) against the
    oracle's state step by step: rows of segment s must be exactly the positions whose KV the oracle lacks there."""
    filled = None
    n_forced = 0
    for before, pend, pos, forced, reached, after in _oracle_run(tau, cap):
        if filled is None:
            filled = list(before)
        assert filled == before
        g_forced, rows, _ = ee.plan(filled, pos, cap)
        assert g_forced == forced == (cap > 0 and pend >= cap)   # a cap <= 0 means none: no step is ever forced
        n_forced += int(forced)
        for s, (lo, hi) in enumerate(rows):
            assert (lo, hi) == (before[s], pos)                  # resume: from where segment s lacks KV up to the current token
        _, rows_rf, _ = ee.plan(filled, pos, cap, refeed=True)
        assert all(r == (before[-1], pos) for r in rows_rf)      # re-feed: every deferred token from layer 1
        assert rows_rf[0][1] - rows_rf[0][0] == pend             # deferred + current = pend + 1 rows
        _, _, filled = ee.plan(filled, pos, cap, reached=reached)
        assert filled == after
    if tau == 0.0:
        assert (n_forced > 0) == (cap > 0)
    # a flush leaves nothing pending
    _, rows, flushed = ee.plan(filled, -1, cap, reached=len(filled) - 1)
    assert all(hi == filled[0] - 1 for _, hi in rows) and flushed == [filled[0]] * len(filled)


def test_step_plan_rejects_bad_state():
    L = ee.lib()
    f = (C.c_int32 * 3)(5, 6, 4)  # watermarks must be non-increasing in depth
    assert L.ee_debug_plan(3, f, 5, 4, 0, -1, None, None, None) == -4
    f = (C.c_int32 * 3)(6, 5, 4)
    assert L.ee_debug_plan(3, f, 6, 4, 0, 3, None, None, None) == -7    # segment out of range
    assert L.ee_debug_plan(3, f, -1, 4, 0, 1, None, None, None) == -7   # a flush ends in the last segment
    assert L.ee_debug_plan(0, f, 6, 4, 0, -1, None, None, None) == -7
    assert L.ee_debug_plan(3, None, 6, 4, 0, -1, None, None, None) == -7
