"""Builds an oracle model from the seeded workload generator (test infrastructure only)."""
from __future__ import annotations

from workload import ModelShape, TensorKind, model_tensor, model_tensor_list, to_numpy  # noqa: F401

from . import oracle as O


def config_of(shape: ModelShape) -> O.EoConfig:
    return O.make_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff,
                         shape.vocab, shape.exit_layers, shape.dtype, shape.rms_eps, shape.rope_base, shape.exit_flags)


def build_model(shape: ModelShape, seed: int = 0, gain_jitter: float = 0.0, layers=None) -> O.Model:
    """All tensors of the seeded model (or only those of the given layers, for spot checks)."""
    m = O.Model(config_of(shape))
    per_layer = (TensorKind.ATTN_NORM, TensorKind.WQ, TensorKind.WK, TensorKind.WV, TensorKind.WO,
                 TensorKind.MLP_NORM, TensorKind.WG, TensorKind.WU, TensorKind.WD)
    for kind, idx in model_tensor_list(shape):
        if layers is not None and kind in per_layer and idx not in layers:
            continue
        m.set_tensor(kind, idx, to_numpy(model_tensor(shape, kind, idx, seed, "cpu", gain_jitter)))
    return m
