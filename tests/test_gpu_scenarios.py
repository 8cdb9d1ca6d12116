"""A serving-like scenario through the C ABI: more requests than sequence slots, so slots are reset and their cache
blocks handed to the next request while the other sequences keep decoding; prompts of 3..90 tokens (short ones through
the decode kernels, long bf16 ones through the prompt-phase GEMMs), deferred-token lists of different lengths in one
step, resume and re-feed modes.  Every request must produce exactly the tokens and exit layers it produces alone in a
fresh cache (the single-sequence path is checked against the CPU oracle by the lockstep tests), and the block pool
must be whole again at the end."""
import numpy as np
import pytest

import paper_2312_04916_amd as ee
from workload import ModelShape, prompt_tokens

from common import load_gpu_model

pytestmark = pytest.mark.gpu

SHAPE = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "f32", 0.02, 0.3)


def _alone(gm, shape, prompt, n_new, tau, cap, refeed):
    cache = ee.KvCache(gm, 1, 256, 32, cap)
    cache.set_refeed(refeed)
    seqs = ee.Sequences(shape.n_layers)
    tok, ex, _ = ee.prefill(gm, cache, 0, prompt, tau)
    seqs.start(0, tok)
    out = [(int(tok), int(ex))]
    for _ in range(n_new - 1):
        ro, tk, pm = seqs.rows([0])
        nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, tau)
        seqs.update([0], nt, exl)
        out.append((int(nt[0]), int(exl[0])))
    cache.close()
    return out


@pytest.mark.parametrize("refeed", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_requests_share_slots_and_blocks(dtype, refeed):
    import dataclasses
    shape = dataclasses.replace(SHAPE, dtype=dtype)
    print(f"case: scenario {dtype} refeed={refeed}", flush=True)
    gm = load_gpu_model(shape, 23, gain_jitter=0.1, max_positions=160, max_rows=64, max_seqs=5)
    rng = np.random.default_rng(7)
    n_jobs, n_slots, tau, cap = 14, 5, 0.12, 5
    jobs = [(prompt_tokens(shape.vocab, int(rng.integers(3, 91)), 300 + j).numpy(), int(rng.integers(5, 31))) for j in range(n_jobs)]
    # a pool that cannot hold five long requests at once were it not for the blocks coming back: 5 slots x 4 blocks
    cache = ee.KvCache(gm, n_slots, 5 * 4 * 32, 32, cap)
    cache.set_refeed(refeed)
    seqs = ee.Sequences(shape.n_layers)
    slot_job = {}
    got = {j: [] for j in range(n_jobs)}
    next_job, layers = 0, set()
    while next_job < n_jobs or slot_job:
        for s in range(n_slots):
            if s not in slot_job and next_job < n_jobs:
                prompt, _ = jobs[next_job]
                tok, ex, _ = ee.prefill(gm, cache, s, prompt, tau)
                seqs.start(s, tok)
                got[next_job].append((int(tok), int(ex)))
                slot_job[s] = next_job
                next_job += 1
        active = sorted(s for s in slot_job if len(got[slot_job[s]]) < jobs[slot_job[s]][1])
        if active:
            ro, tk, pm = seqs.rows(active)
            nt, exl, _ = ee.decode_step(gm, cache, active, ro, tk, pm, tau)
            seqs.update(active, nt, exl)
            for i, s in enumerate(active):
                got[slot_job[s]].append((int(nt[i]), int(exl[i])))
                layers.add(int(exl[i]))
        for s in list(slot_job):
            if len(got[slot_job[s]]) >= jobs[slot_job[s]][1]:
                cache.reset(s)
                del slot_job[s]
    assert len(layers) >= 2, layers
    # the pool is whole again: five fresh requests of four blocks each fit
    for s in range(n_slots):
        ee.prefill(gm, cache, s, prompt_tokens(shape.vocab, 100, 900 + s).numpy(), 1.0)
    cache.close()
    for j, (prompt, n_new) in enumerate(jobs):
        assert got[j] == _alone(gm, shape, prompt, n_new, tau, cap, refeed), j
    gm.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_steps_on_alternating_streams_equal_one_stream(dtype):
    """A decode step with one sequence leaves two kernels of the next layer in flight when its token takes an exit;
    the next call may come on another stream and must be ordered behind them.  Steps issued on two streams in turn
    (with a cache read on a third in between) must give the tokens, exit layers and cache of the same steps on one
    stream."""
    import dataclasses
    import torch
    shape = dataclasses.replace(SHAPE, dtype=dtype)
    gm = load_gpu_model(shape, 3, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=1)
    prompt = prompt_tokens(shape.vocab, 21, 8).numpy()
    tau, n_new = 0.004, 40  # low threshold: most tokens leave at the first exit

    def run(streams):
        cache = ee.KvCache(gm, 1, 256, 32, 15)
        seqs = ee.Sequences(shape.n_layers)
        tok, ex, _ = ee.prefill(gm, cache, 0, prompt, tau, stream=streams[0])
        seqs.start(0, tok)
        out = [(int(tok), int(ex))]
        for i in range(n_new - 1):
            ro, tk, pm = seqs.rows([0])
            nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, tau, stream=streams[i % len(streams)])
            seqs.update([0], nt, exl)
            out.append((int(nt[0]), int(exl[0])))
            if i % 7 == 3:
                cache.read(0, 0, 0, 5, stream=streams[-1])
        cache.flush([0], stream=streams[0])
        kv = [cache.read(0, l, 0, len(prompt) + n_new - 1, stream=streams[-1]) for l in range(shape.n_layers)]
        cache.close()
        return out, kv

    try:
        one = torch.cuda.Stream()
        ref_out, ref_kv = run([one])
        assert sum(1 for _, e in ref_out if e < shape.n_layers) >= n_new // 2, ref_out
        out, kv = run([torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()])
        assert out == ref_out
        for (k, v), (k0, v0) in zip(kv, ref_kv):
            assert np.array_equal(k, k0) and np.array_equal(v, v0)
    finally:
        gm.close()
