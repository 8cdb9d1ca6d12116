"""ee_decode_step_static (the decode step whose workspace is an array the library keeps in the GPU's memory, for
callers that cannot allocate) against ee_decode_step through the C ABI: the same model drives two caches in the same
state, one through each entry point; tokens, exit layers and confidences must be identical bit for bit, step after
step, on a call with two sequences and their deferred rows and then on a smaller call with one sequence, and the
caches must hold the same K and V afterwards.  Also: a model whose decode workspace exceeds the array is refused."""
import dataclasses

import numpy as np
import pytest

import paper_2312_04916_amd as ee
from workload import CONFIGS, ModelShape, prompt_tokens

from common import load_gpu_model

pytestmark = pytest.mark.gpu

TINY = {"f32": CONFIGS["C1"].shape, "bf16": ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "bf16", 0.02, 0.3)}


def _drive(gm, shape, prompts, tau, cap, n_build, max_tokens):
    """Two caches brought to the same state with ee_decode_step (n_build steps, so that lists of deferred tokens
    exist), then: a step over both sequences, a step over sequence 0 alone, and a few more alternating ones, cache A
    through ee_decode_step and cache B through ee_decode_step_static."""
    ids = list(range(len(prompts)))
    caches = [ee.KvCache(gm, len(ids), max_tokens, 32, cap) for _ in range(2)]
    seqs = [ee.Sequences(shape.n_layers) for _ in range(2)]
    for cache, sq in zip(caches, seqs):
        for s in ids:
            tok, _, _ = ee.prefill(gm, cache, s, prompts[s], tau)
            sq.start(s, tok)
        for _ in range(n_build):
            ro, tk, pm = sq.rows(ids)
            nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
            sq.update(ids, nt, exl)
    assert seqs[0].pending == seqs[1].pending and seqs[0].current == seqs[1].current
    rows_seen = []
    for which in (ids, ids[:1], ids, ids[:1], ids[1:], ids):
        outs = []
        for k, (cache, sq) in enumerate(zip(caches, seqs)):
            ro, tk, pm = sq.rows(which)
            nt, exl, cf = ee.decode_step(gm, cache, which, ro, tk, pm, tau, static_workspace=(k == 1))
            sq.update(which, nt, exl)
            outs.append((nt.copy(), exl.copy(), cf.copy()))
            if k == 1:
                rows_seen.append(len(tk))
        a, b = outs
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), (which, a, b)
        assert np.array_equal(a[2].view(np.int32), b[2].view(np.int32)), (which, a[2], b[2])
    for cache in caches:
        cache.flush(ids)
    for s in ids:
        n_pos = caches[0].filled(s, 0)
        assert n_pos == caches[1].filled(s, 0)
        for l in range(shape.n_layers):
            ka, va = caches[0].read(s, l, 0, n_pos)
            kb, vb = caches[1].read(s, l, 0, n_pos)
            assert np.array_equal(ka, kb) and np.array_equal(va, vb), (s, l)
    for cache in caches:
        cache.close()
    return rows_seen


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_workspace_step_equals_decode_step_tiny(dtype):
    shape = TINY[dtype]
    print(f"case: static workspace, tiny {dtype}", flush=True)
    gm = load_gpu_model(shape, 0, gain_jitter=0.1, max_positions=128, max_rows=64, max_seqs=2)
    prompts = [prompt_tokens(shape.vocab, 16, 1).numpy(), prompt_tokens(shape.vocab, 23, 2).numpy()]
    try:
        rows = _drive(gm, shape, prompts, 0.0, 8, 5, 512)   # every token leaves at the first exit: 5 deferred each
        assert rows[:2] == [12, 7], rows                     # two sequences with their lists, then one: a smaller call
        _drive(gm, shape, prompts, 0.35, 8, 5, 512)          # a mix of exits, heads that do not fire
    finally:
        gm.close()


def test_static_workspace_step_at_the_7b_widths_and_size_limit():
    """Two layers of the 7B widths with max_rows 64: the decode workspace (28 MB) nearly fills the 32 MB array.  The
    same widths with max_rows 256 need 100 MB and are refused before anything is touched."""
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,))
    print("case: static workspace, 7B widths", flush=True)
    gm = load_gpu_model(shape, 0, max_positions=256, max_rows=64, max_seqs=2)
    prompts = [prompt_tokens(shape.vocab, 70, 1).numpy(), prompt_tokens(shape.vocab, 40, 2).numpy()]
    try:
        rows = _drive(gm, shape, prompts, 0.0, 15, 4, 1024)
        assert rows[:2] == [10, 6], rows
        _drive(gm, shape, prompts, 0.12, 15, 4, 1024)
    finally:
        gm.close()
    big = ee.Model(ee.config_of_shape(shape, 256), 256, 16)      # no tensors needed: the size is checked first
    cache = ee.KvCache(big, 1, 256, 32, 15)
    with pytest.raises(ee.EeError) as e:
        ee.decode_step(big, cache, [0], [0, 1], [1], [0], 0.5, static_workspace=True)
    assert e.value.code == -2
    cache.close()
    big.close()
