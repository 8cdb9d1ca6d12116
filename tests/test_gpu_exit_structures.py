"""GPU parity of the exit structures of Section 2 ("Model architectures": exits without a normalisation, tied
input/output embeddings, an MLP in front of the exit's output embedding), through the C ABI, against the CPU
oracle: generation in lockstep (tokens and exit layers exact outside the guard band, hidden states, head logits
and confidences within 1e-4 for fp32 and 2e-3 for bf16), batches against each sequence alone, the weight file,
and the prompt-phase GEMM path with the heads scored on every position."""
import dataclasses
import os
import tempfile

import numpy as np
import pytest

import paper_2312_04916_amd as ee
from oracle.from_workload import build_model
from workload import ModelShape, TensorKind, model_tensor, prompt_tokens, write_weight_file

from common import GUARD, TOL, TOL_CONF, ee_config_of, kv_check, load_gpu_model, lockstep, rel_err

pytestmark = pytest.mark.gpu

BASE = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "f32", 0.02, 0.3)
VARIANTS = {
    "no_norm": dict(exit_norm=False),
    "tied": dict(tie_embeddings=True, head_sigma=0.5),
    "mlp": dict(exit_mlp=True),
    "all": dict(exit_norm=False, tie_embeddings=True, exit_mlp=True, head_sigma=0.5),
}


def shape_of(name, dtype):
    return dataclasses.replace(BASE, dtype=dtype, **VARIANTS[name])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", list(VARIANTS))
def test_lockstep_generation_with_other_exit_structures(name, dtype):
    shape = shape_of(name, dtype)
    om = build_model(shape, 11, gain_jitter=0.1)
    gm = load_gpu_model(shape, 11, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=2)
    prompt = prompt_tokens(shape.vocab, 40 if dtype == "bf16" else 16, 12).numpy()  # bf16: the prompt-phase GEMM path
    exits_seen = set()
    for tau in (0.0, 0.1, 0.3, 1.0):
        print(f"case: exit structure {name} {dtype} tau={tau}", flush=True)
        cache = ee.KvCache(gm, 2, 512, 32, 6)
        logits = gm.enable_logits(1)
        rep = lockstep(gm, cache, om, prompt, 24, tau, max_pending=6, logits=logits)
        assert not rep.mismatches, rep.mismatches[:5]
        assert rep.max_hidden_err <= TOL[dtype], rep.max_hidden_err
        assert rep.max_logit_err <= TOL[dtype], rep.max_logit_err
        assert rep.max_conf_err <= TOL_CONF[dtype], rep.max_conf_err
        exits_seen.update(rep.exit_layers)
        if tau == 0.0:
            assert rep.forced_full > 0  # the cap of 6 forces full-depth steps: the deferred rows pass the exits untouched
        # after a flush the cache equals a full-depth forward of the whole sequence (the exits' MLPs left no trace)
        cache.flush([0])
        seq = np.concatenate([prompt, np.array(rep.tokens[:-1], np.int32)])
        _, ko, vo = om.forward_sequence(seq)
        for l in range(shape.n_layers):
            k, v = cache.read(0, l, 0, len(seq))
            kv_check(k, ko[l], dtype, "K", l), kv_check(v, vo[l], dtype, "V", l)
        cache.close()
    assert len(exits_seen) >= 2, exits_seen
    gm.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batch_of_20_with_exit_mlps_equals_each_alone(dtype):
    """Twenty sequences in one step: the exits' MLPs and heads run over 20 rows (more than one MFMA row tile, the
    packed-operand variants for bf16); every sequence must emit what it emits alone."""
    shape = shape_of("all", dtype)
    print(f"case: exit structures batch {dtype}", flush=True)
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

    both = run(list(range(n_seq)))
    layers = set()
    for s in range(n_seq):
        assert both[s] == run([s])[s], s
        layers.update(e for _, e in both[s])
    assert len(layers) >= 2, layers
    gm.close()


def test_weight_file_with_exit_flags_and_tensor_checks():
    shape = shape_of("all", "bf16")
    prompt = prompt_tokens(shape.vocab, 12, 3).numpy()
    gm = load_gpu_model(shape, 5, gain_jitter=0.1, max_positions=64, max_rows=16, max_seqs=1)
    cache = ee.KvCache(gm, 1, 128, 32, 4)
    ref = ee.prefill(gm, cache, 0, prompt, 0.1)
    # tensors the configured structure does not have are refused
    for kind in (TensorKind.EXIT_NORM, TensorKind.EXIT_HEAD, TensorKind.FINAL_HEAD):
        t = model_tensor(dataclasses.replace(BASE, dtype="bf16"), kind, 0, 5, "cuda:0", 0.1).contiguous()
        with pytest.raises(ee.EeError) as e:
            gm.set_tensor(int(kind), 0, t)
        assert e.value.code == -1
    cache.close()
    gm.close()
    with tempfile.TemporaryDirectory() as td:
        path = os.path.join(td, "w.bin")
        write_weight_file(path, shape, 5, 64, gain_jitter=0.1)
        assert open(path, "rb").read(8) == b"EEWT0002"
        gm2 = ee.model_load(ee_config_of(shape, 64), path, 16, 1)
        cache = ee.KvCache(gm2, 1, 128, 32, 4)
        got = ee.prefill(gm2, cache, 0, prompt, 0.1)
        assert got[0] == ref[0] and got[1] == ref[1] and np.allclose(got[2], ref[2], atol=1e-6)
        cache.close()
        gm2.close()
        # a file of another structure is refused
        with pytest.raises(ee.EeError) as e:
            ee.model_load(ee_config_of(shape_of("mlp", "bf16"), 64), path, 16, 1)
        assert e.value.code == -5
    # a model without an exit MLP does not have its tensors
    gm3 = load_gpu_model(shape_of("tied", "bf16"), 5, gain_jitter=0.1, max_positions=64, max_rows=16, max_seqs=1)
    t = model_tensor(shape, TensorKind.EXIT_WD, 0, 5, "cuda:0").contiguous()
    with pytest.raises(ee.EeError) as e:
        gm3.set_tensor(int(TensorKind.EXIT_WD), 0, t)
    assert e.value.code == -1
    gm3.close()


@pytest.mark.parametrize("name", list(VARIANTS))
def test_scored_prompt_phase_with_other_exit_structures(name):
    """Every head on every prompt position through the prompt-phase GEMMs (bf16, d_model = 256)."""
    shape = dataclasses.replace(ModelShape(3, 256, 4, 64, 512, 2048, (1, 2), "bf16", 0.02, 0.3 / 2 ** 0.5), **VARIANTS[name])
    print(f"case: scored prompt phase {name}", flush=True)
    om = build_model(shape, 21, gain_jitter=0.1)
    gm = load_gpu_model(shape, 21, gain_jitter=0.1, max_positions=512, max_rows=64, max_seqs=1, scored_head_terms=2)
    n = 150
    p = prompt_tokens(shape.vocab, n, 22).numpy()
    cache = ee.KvCache(gm, 1, 512, 64, 8)
    hid, ko, vo = om.forward_sequence(p)
    tok, ex, conf, ptok, pconf = ee.prefill_scored(gm, cache, 0, p, 0.3)
    for l in range(shape.n_layers):
        k, v = cache.read(0, l, 0, n)
        kv_check(k, ko[l], "bf16", "K", l), kv_check(v, vo[l], "bf16", "V", l)
    heads = list(shape.exit_layers) + [shape.n_layers]
    for hi, layer in enumerate(heads):
        for pos in range(n):
            _, dg = om.head_row(hi, hid[layer][pos])
            if int(ptok[hi, pos]) != dg["argmax"]:
                assert dg["top1"] - dg["top2"] < GUARD and int(ptok[hi, pos]) == dg["arg2"], (hi, pos)
            assert abs(float(pconf[hi, pos]) - dg["conf"]) <= TOL_CONF["bf16"], (hi, pos, float(pconf[hi, pos]), dg["conf"])
    cache.close()
    gm.close()


def test_plain_prompt_phase_runs_the_exit_mlps_on_the_last_position():
    """The plain entry point evaluates the exits on the last position only: their MLPs run through the decode
    kernels on a copy of that row."""
    shape = dataclasses.replace(ModelShape(3, 256, 4, 64, 512, 2048, (1, 2), "bf16", 0.02, 0.3 / 2 ** 0.5), exit_mlp=True)
    print("case: plain prompt phase with exit MLPs", flush=True)
    gm = load_gpu_model(shape, 21, gain_jitter=0.1, max_positions=128, max_rows=16, max_seqs=1)
    cache = ee.KvCache(gm, 1, 128, 64, 8)
    om = build_model(shape, 21, gain_jitter=0.1)
    p = prompt_tokens(shape.vocab, 40, 1).numpy()
    tok, ex, conf = ee.prefill(gm, cache, 0, p, 0.3)
    hid, _, _ = om.forward_sequence(p)
    for hi, layer in enumerate(list(shape.exit_layers) + [shape.n_layers]):
        _, dg = om.head_row(hi, hid[layer][-1])
        assert abs(float(conf[hi]) - dg["conf"]) <= TOL_CONF["bf16"], (hi, float(conf[hi]), dg["conf"])
    assert rel_err(cache.read_hidden(0), hid[shape.n_layers][-1]) <= TOL["bf16"]
    cache.close()
    gm.close()
