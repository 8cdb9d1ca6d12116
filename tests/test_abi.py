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
