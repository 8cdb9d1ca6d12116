"""GPU parity on shapes off the beaten track, through the C ABI, against the CPU oracle: widths that are not a
power of two (three heads), feed-forward and vocabulary sizes that leave ragged tile groups, a model without
exits, a model with an exit after every layer, a single head of 128.  Generation in lockstep (tokens and exit
layers exact outside the guard band; hidden states, logits and confidences within 1e-4 for fp32 and 2e-3 for
bf16), then the flushed cache against a full-depth forward of the whole sequence (Section 5.2: KV recomputation
leaves the cache a full-depth pass would have written)."""
import numpy as np
import pytest

import paper_2312_04916_amd as ee
from oracle.from_workload import build_model
from workload import ModelShape, prompt_tokens

from common import TOL, TOL_CONF, kv_check, load_gpu_model, lockstep, rel_err

pytestmark = pytest.mark.gpu

SHAPES = {
    # 3 heads of 32: d = 96 (3 k-tiles), 5 tiles of gate and up, 34 vocabulary tiles
    "d96": ModelShape(3, 96, 3, 32, 160, 544, (1,), "f32", 0.02, 0.35),
    # 3 heads of 64, no exit at all: plain full-depth decoding through the same entry points
    "d192_no_exits": ModelShape(2, 192, 3, 64, 224, 1056, (), "f32", 0.02, 0.3),
    # one head of 128, an exit after every layer but the last, a vocabulary of three tiles
    "one_head_all_exits": ModelShape(5, 128, 1, 128, 96, 96, (1, 2, 3, 4), "f32", 0.02, 0.6),
}


def shape_of(name, dtype):
    import dataclasses
    return dataclasses.replace(SHAPES[name], dtype=dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_lockstep_generation_on_odd_shapes(name, dtype):
    shape = shape_of(name, dtype)
    om = build_model(shape, 17, gain_jitter=0.1)
    gm = load_gpu_model(shape, 17, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=1)
    # 70 tokens: bf16 models whose width allows it take the prompt-phase GEMM path with a ragged last row tile
    prompt = prompt_tokens(shape.vocab, 70, 18).numpy()
    exits_seen = set()
    for tau in (0.0, 0.15, 0.4, 1.0):
        print(f"case: odd shape {name} {dtype} tau={tau}", flush=True)
        cache = ee.KvCache(gm, 1, 256, 32, 5)
        logits = gm.enable_logits(1)
        rep = lockstep(gm, cache, om, prompt, 20, tau, max_pending=5, logits=logits)
        assert not rep.mismatches, rep.mismatches[:5]
        assert rep.max_hidden_err <= TOL[dtype], rep.max_hidden_err
        assert rep.max_logit_err <= TOL[dtype], rep.max_logit_err
        assert rep.max_conf_err <= TOL_CONF[dtype], rep.max_conf_err
        exits_seen.update(rep.exit_layers)
        cache.flush([0])
        seq = np.concatenate([prompt, np.array(rep.tokens[:-1], np.int32)])
        _, ko, vo = om.forward_sequence(seq)
        for l in range(shape.n_layers):
            k, v = cache.read(0, l, 0, len(seq))
            kv_check(k, ko[l], dtype, "K", l), kv_check(v, vo[l], dtype, "V", l)
        cache.close()
    if shape.exit_layers:
        assert len(exits_seen) >= 2, exits_seen
    else:
        assert exits_seen == {shape.n_layers}
    gm.close()
