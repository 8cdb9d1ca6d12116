"""GPU parity of exits that contain a complete Transformer layer (Section 2, "Model architectures"; Appendix D.1),
through the C ABI, against the CPU oracle: generation in lockstep, the backbone's cache and the exit layers' own
caches after a flush, re-feed and pipeline modes, a batch against each sequence alone, the weight file, and the 7B
widths."""
import dataclasses
import os
import tempfile

import numpy as np
import pytest

import paper_2312_04916_amd as ee
from oracle.from_workload import build_model
from workload import CONFIGS, ModelShape, prompt_tokens, write_weight_file

from common import TOL, TOL_CONF, build_pair, ee_config_of, kv_check, load_gpu_model, lockstep

pytestmark = pytest.mark.gpu

BASE = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "f32", 0.02, 0.3, exit_layer=True)


def _check_caches(cache, om, shape, seq_tokens):
    """Backbone layers against the oracle's cache-free forward; the layer inside exit i (cache layer L + i) against
    the oracle's exit layer applied to the hidden states at the exit's depth."""
    n = len(seq_tokens)
    hid, ko, vo = om.forward_sequence(seq_tokens)
    for l in range(shape.n_layers):
        assert cache.filled(0, l) == n
        k, v = cache.read(0, l, 0, n)
        kv_check(k, ko[l], shape.dtype, "K", l), kv_check(v, vo[l], shape.dtype, "V", l)
    for e, layer in enumerate(shape.exit_layers):
        assert cache.filled(0, shape.n_layers + e) == n
        _, ke, ve = om.exit_layer_sequence(e, hid[layer])
        k, v = cache.read(0, shape.n_layers + e, 0, n)
        kv_check(k, ke, shape.dtype, "K (exit layer)", layer), kv_check(v, ve, shape.dtype, "V (exit layer)", layer)


@pytest.mark.parametrize("mode", ["resume", "refeed", "pipeline"])
@pytest.mark.parametrize("dtype,n_prompt", [("f32", 16), ("bf16", 16), ("bf16", 40)])
def test_lockstep_generation_with_exit_layers(dtype, n_prompt, mode):
    shape = dataclasses.replace(BASE, dtype=dtype)
    om = build_model(shape, 11, gain_jitter=0.1)
    gm = load_gpu_model(shape, 11, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=2)
    prompt = prompt_tokens(shape.vocab, n_prompt, 12).numpy()  # 40 bf16 tokens: the prompt-phase GEMM path
    exits_seen = set()
    try:
        for tau in (0.0, 0.1, 0.3, 1.0):
            print(f"case: exit layer {dtype} prompt {n_prompt} {mode} tau={tau}", flush=True)
            cache = ee.KvCache(gm, 2, 512, 32, 6)
            if mode == "refeed":
                cache.set_refeed(True)
            if mode == "pipeline":
                cache.set_pipeline(True)
            logits = gm.enable_logits(1)
            cap = 0 if mode == "pipeline" else 6
            rep = lockstep(gm, cache, om, prompt, 22, tau, max_pending=cap, logits=logits, pipeline=(mode == "pipeline"))
            assert not rep.mismatches, rep.mismatches[:5]
            assert rep.max_hidden_err <= TOL[dtype], rep.max_hidden_err
            assert rep.max_logit_err <= TOL[dtype], rep.max_logit_err
            assert rep.max_conf_err <= TOL_CONF[dtype], rep.max_conf_err
            exits_seen.update(rep.exit_layers)
            if tau == 0.0 and mode != "pipeline":
                assert rep.forced_full > 0  # forced steps: their rows still leave K and V in the exits' layers
            cache.flush([0])
            _check_caches(cache, om, shape, np.concatenate([prompt, np.array(rep.tokens[:-1], np.int32)]))
            cache.close()
        assert len(exits_seen) >= 2, exits_seen
    finally:
        gm.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batch_of_20_with_exit_layers_equals_each_alone(dtype):
    """Twenty sequences in one step: the exits' layers run over all the rows of the step (20 current tokens plus the
    deferred ones: packed operands for bf16, several attention query tiles); every sequence emits what it emits alone."""
    shape = dataclasses.replace(BASE, dtype=dtype)
    print(f"case: exit layer batch {dtype}", flush=True)
    gm = load_gpu_model(shape, 13, gain_jitter=0.1, max_positions=128, max_rows=256, max_seqs=20)
    n_seq, n_new, tau, cap = 20, 10, 0.12, 7
    prompts = [prompt_tokens(shape.vocab, 5 + s, 30 + s).numpy() for s in range(n_seq)]

    def run(ids):
        cache = ee.KvCache(gm, n_seq, 4096, 32, cap)
        seqs = ee.Sequences(shape.n_layers)
        out = {s: [] for s in ids}
        for s in ids:
            tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], tau)
            seqs.start(s, tok)
            out[s].append((int(tok), int(ex)))
        for _ in range(n_new - 1):
            ro, tk, pm = seqs.rows(ids)
            nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
            seqs.update(ids, nt, exl)
            for j, s in enumerate(ids):
                out[s].append((int(nt[j]), int(exl[j])))
        cache.close()
        return out

    try:
        both = run(list(range(n_seq)))
        layers = set()
        for s in range(n_seq):
            assert both[s] == run([s])[s], s
            layers.update(e for _, e in both[s])
        assert len(layers) >= 2, layers
    finally:
        gm.close()


def test_exit_layer_weight_file_and_refusals():
    shape = dataclasses.replace(BASE, dtype="bf16")
    prompt = prompt_tokens(shape.vocab, 40, 3).numpy()
    gm = load_gpu_model(shape, 5, gain_jitter=0.1, max_positions=64, max_rows=16, max_seqs=1)
    cache = ee.KvCache(gm, 1, 128, 32, 4)
    ref = ee.prefill(gm, cache, 0, prompt, 0.1)
    cache.reset(0)
    with pytest.raises(ee.EeError) as e:  # the scored prompt phase does not run the exits' layers
        ee.prefill_scored(gm, cache, 0, prompt, 0.1)
    assert e.value.code == -1
    cache.close()
    gm.close()
    with tempfile.TemporaryDirectory() as td:
        path = os.path.join(td, "w.bin")
        write_weight_file(path, shape, 5, 64, gain_jitter=0.1)
        gm2 = ee.model_load(ee_config_of(shape, 64), path, 16, 1)
        cache = ee.KvCache(gm2, 1, 128, 32, 4)
        got = ee.prefill(gm2, cache, 0, prompt, 0.1)
        assert got[0] == ref[0] and got[1] == ref[1] and np.allclose(got[2], ref[2], atol=1e-6)
        cache.close()
        gm2.close()
    both = dataclasses.replace(shape, exit_mlp=True)  # an MLP of its own and a layer of its own: not a configuration
    with pytest.raises(ee.EeError) as e:
        ee.Model(ee_config_of(both, 64), 16, 1)
    assert e.value.code == -1


def test_exit_layer_at_the_7b_widths():
    """Two layers of the 7B widths with a third, full-width layer inside the exit; 48-token prompt through the
    prompt-phase GEMMs (which fill the exit layer's cache), decode steps with deferred rows.  Lockstep with the oracle."""
    from oracle import oracle as O
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,), exit_layer=True)
    print("case: exit layer, 7B widths", flush=True)
    O.set_threads(16)
    om, gm = build_pair(shape, 0, max_positions=128)
    prompt = prompt_tokens(shape.vocab, 48, 1).numpy()
    try:
        cache = ee.KvCache(gm, 1, 128, 64, 15)
        logits = gm.enable_logits(1)
        rep = lockstep(gm, cache, om, prompt, 14, 0.12, max_pending=15, logits=logits)
        print(f"  exits {rep.exit_layers} teacher-forced {rep.teacher_forced} hidden {rep.max_hidden_err:.2e} "
              f"logits {rep.max_logit_err:.2e}", flush=True)
        assert not rep.mismatches, rep.mismatches[:5]
        assert rep.max_hidden_err <= TOL["bf16"] and rep.max_logit_err <= TOL["bf16"] and rep.teacher_forced <= 2
        cache.flush([0])
        _check_caches(cache, om, shape, np.concatenate([prompt, np.array(rep.tokens[:-1], np.int32)]))
        cache.close()
    finally:
        gm.close()
        O.set_threads(1)
