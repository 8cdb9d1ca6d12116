"""GPU parity at the real shapes of the benchmark workloads (C2 1.3B-shaped, C3 7B-shaped), through the C ABI,
in the launch configuration bench.py times (batch 1, 64-token cache blocks, max_pending 15).

Where the oracle can follow in seconds (reduced prompt / few layers) the check is the lockstep comparison;
at the full 32-layer depth and 1024-token context it is the paper's invariants, which hold at any size:
threshold 1 never exits, threshold 0 always exits at the first exit (up to the forced full passes), and after
generation + flush the KV cache equals a full-depth prefill of the generated sequence (Section 4)."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2312_04916_amd as ee
from oracle import oracle as O
from workload import ModelShape, CONFIGS, prompt_tokens

from common import TOL, tol_for, TOL_CONF, build_pair, kv_check, load_gpu_model, lockstep, rel_err

pytestmark = pytest.mark.gpu

TOL = TOL["bf16"]  # hidden states, logits, confidences (relative to the largest reference magnitude)


def _lockstep_case(shape, n_prompt, n_new, taus, prompt_seed=1, want_deferred=False):
    O.set_threads(16)
    om, gm = build_pair(shape, 0, max_positions=n_prompt + n_new + 8)
    prompt = prompt_tokens(shape.vocab, n_prompt, prompt_seed).numpy()
    logits = gm.enable_logits(1)
    try:
        for tau in taus:
            print(f"case: lockstep d={shape.d_model} L={shape.n_layers} prompt {n_prompt} tau {tau}", flush=True)
            cache = ee.KvCache(gm, 1, n_prompt + n_new + 8, 64, 15)
            rep = lockstep(gm, cache, om, prompt, n_new, tau, max_pending=15, logits=logits)
            print(f"  exits {sorted(set(rep.exit_layers))} teacher-forced {rep.teacher_forced} hidden {rep.max_hidden_err:.2e} "
                  f"logits {rep.max_logit_err:.2e} conf {rep.max_conf_err:.2e}", flush=True)
            assert not rep.mismatches, rep.mismatches[:5]
            tol = tol_for(shape)
            assert rep.max_hidden_err <= tol and rep.max_logit_err <= tol and rep.max_conf_err <= TOL_CONF["bf16"]
            assert rep.teacher_forced <= max(2, n_new // 8)
            if want_deferred:
                deferred_steps = sum(1 for j in range(1, n_new) if rep.exit_layers[j - 1] != shape.n_layers)
                assert deferred_steps >= 2 and shape.n_layers in rep.exit_layers[1:], rep.exit_layers
            n_pos = n_prompt + n_new - 1
            cache.flush([0])
            rep.state.flush()
            for l in sorted({0, shape.exit_layers[0] if shape.exit_layers else 0, shape.n_layers - 1}):
                k, v = cache.read(0, l, 0, n_pos)
                ko, vo = rep.state.kv_read(l, 0, n_pos)
                kv_check(k, ko, "bf16", "K", l), kv_check(v, vo, "bf16", "V", l)
            cache.close()
    finally:
        gm.close()
        O.set_threads(1)


def test_c2_shape_lockstep_reduced_prompt():
    """1.3B-shaped model, all 24 layers; prompt cut to 96 tokens, 40 new tokens."""
    _lockstep_case(CONFIGS["C2"].shape, 96, 40, (0.2, 0.8))


def test_c3_shape_two_layers_long_context():
    """7B-shaped layers and heads (every kernel in its benchmark launch shape), 2 layers, context 333+."""
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,))
    _lockstep_case(shape, 333, 20, (0.2,))


def test_c3_benchmark_launch_shape_context_1024():
    """The launch shape bench.py times at the 7B widths: batch 1, a 1024-token prompt (so the decode attention runs as
    workgroups of 8 waves over several KV splits that the O projection merges), 64-token blocks, max_pending 15;
    2 layers with the exit between them, so steps carry deferred rows.  Lockstep against the oracle."""
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,))
    _lockstep_case(shape, CONFIGS["C3"].prompt_len[0], 14, (0.12,), want_deferred=True)


def test_c5_widths_one_layer_context_2048():
    """One layer of the 30B widths (d = 6656, 52 heads of 128) over a 2048-token context, the prompt length of that
    workload: QKV, attention over 2048 positions and the O projection in their real launch shapes, against the oracle.
    d_ff is cut to 2048 to keep the oracle's prompt pass to seconds (the MLP kernels do not depend on the context and
    run at their real width in test_c5_shape_two_layers); no exits, every step runs to full depth."""
    shape = dataclasses.replace(CONFIGS["C5"].shape, n_layers=1, exit_layers=(), d_ff=2048)
    _lockstep_case(shape, CONFIGS["C5"].prompt_len[0], 6, (1.0,))


def test_context_of_4200_positions_small_model():
    """A prompt of 4200 tokens (three passes of the prompt phase, the later ones attending to what the earlier ones
    cached; 66 cache blocks) and decode steps over that context: head_dim 128, two heads, so a step's attention runs
    with the largest number of KV splits and the O projection merges all of them."""
    shape = ModelShape(2, 256, 2, 128, 544, 2080, (1,), "bf16", 0.02, 0.3 / 2 ** 0.5)
    _lockstep_case(shape, 4200, 12, (0.5,))


def test_c5_shape_two_layers():
    """30B-shaped layers and heads (d = 6656, 52 heads, d_ff = 17920: widths that are not powers of two), 2 layers;
    the prompt of 72 tokens goes through the prompt-phase GEMMs, the steps through the decode kernels."""
    shape = dataclasses.replace(CONFIGS["C5"].shape, n_layers=2, exit_layers=(1,))
    _lockstep_case(shape, 72, 12, (0.2,))


def test_c3_shape_exit_mlp_and_tied_embeddings():
    """7B widths, 2 layers, the exit with an MLP of its own and no norm, every head tied to the embedding."""
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,), exit_norm=False, tie_embeddings=True,
                                exit_mlp=True, head_sigma=0.1)
    _lockstep_case(shape, 48, 12, (0.05,))


def test_c3_full_depth_reduced_prompt():
    """The full 7B-shaped model (32 layers, exits after 8 and 16) against the oracle: prompt 24, 12 new tokens."""
    _lockstep_case(CONFIGS["C3"].shape, 24, 12, (0.2,))


def test_c3_full_size_invariants():
    """C3 as benchmarked: prompt 1024, batch 1, 64-token blocks, max_pending 15."""
    wl = CONFIGS["C3"]
    shape, n_prompt, n_new = wl.shape, wl.prompt_len[0], 48
    gm = load_gpu_model(shape, wl.weight_seed, max_positions=n_prompt + n_new + 8, max_rows=64, max_seqs=2)
    prompt = prompt_tokens(shape.vocab, n_prompt, wl.prompt_seed).numpy()
    cache = ee.KvCache(gm, 2, 2 * (n_prompt + n_new + 8), 64, 15)
    L, e1 = shape.n_layers, shape.exit_layers[0]

    def run(tau):
        cache.reset(0)
        tok, ex, _ = ee.prefill(gm, cache, 0, prompt, tau)
        seqs = ee.Sequences(L)
        seqs.start(0, tok)
        toks, exits = [tok], [ex]
        for _ in range(n_new - 1):
            ro, tk, pm = seqs.rows([0])
            nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, tau)
            seqs.update([0], nt, exl)
            toks.append(int(nt[0]))
            exits.append(int(exl[0]))
            assert cache.pending(0) == len(seqs.pending[0]) <= 15
        return toks, exits

    try:
        print("case: C3 full size tau 1.0", flush=True)
        t1, x1 = run(1.0)
        assert set(x1) == {L}
        t1b, _ = run(1.0)
        assert t1 == t1b, "two runs must be bit-identical (fixed-order reductions)"
        print("case: C3 full size tau 0.0", flush=True)
        t0, x0 = run(0.0)
        # token 0 from prefill, then 15 early exits, then one forced full-depth step, repeating
        assert x0[0] == e1 and all(x0[j] == (L if j % 16 == 0 else e1) for j in range(1, n_new))
        print("case: C3 full size tau 0.2 + KV invariant", flush=True)
        toks, exits = run(0.2)
        assert len(set(exits)) >= 2, exits
        cache.flush([0])
        n_pos = n_prompt + n_new - 1
        seq = np.concatenate([prompt, np.array(toks[:-1], np.int32)])
        cache.reset(1)
        ee.prefill(gm, cache, 1, seq, 1.0)
        for l in (0, 7, 8, 15, 16, 31):
            assert cache.filled(0, l) == n_pos and cache.filled(1, l) == n_pos
            k0, v0 = cache.read(0, l, n_prompt - 8, n_new + 7)
            k1, v1 = cache.read(1, l, n_prompt - 8, n_new + 7)
            kv_check(k0, k1, "bf16", "K", l), kv_check(v0, v1, "bf16", "V", l)
    finally:
        cache.close()
        gm.close()


def test_c4_full_size_batch_invariants():
    """C4 as benchmarked (the full 7B-shaped model, 16 ragged sequences, threshold 0.6, max_pending 15, 256 rows per
    launch at most): sampled sequences must emit exactly what they emit alone, and after a flush the cache of a
    sampled sequence equals a full-depth prompt phase over what it generated (Section 4: no KV entry is missing)."""
    from workload import prompt_lengths
    wl = CONFIGS["C4"]
    shape, B, n_new, tau = wl.shape, wl.batch, 24, wl.thresholds[0]
    lens = prompt_lengths(B, wl.prompt_len[0], wl.prompt_len[1], wl.length_seed)
    prompts = [prompt_tokens(shape.vocab, lens[b], wl.prompt_seed + b).numpy() for b in range(B)]
    gm = load_gpu_model(shape, wl.weight_seed, max_positions=max(lens) + n_new + 8, max_rows=256, max_seqs=B)
    cache = ee.KvCache(gm, B + 1, sum(lens) + max(lens) + (B + 1) * (n_new + 72), 64, 15)
    L = shape.n_layers

    def run(ids):
        seqs = ee.Sequences(L)
        out = {s: ([], []) for s in ids}
        for s in ids:
            cache.reset(s)
            tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], tau)
            seqs.start(s, tok)
            out[s][0].append(int(tok))
            out[s][1].append(int(ex))
        for _ in range(n_new - 1):
            ro, tk, pm = seqs.rows(ids)
            nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
            seqs.update(ids, nt, exl)
            for j, s in enumerate(ids):
                out[s][0].append(int(nt[j]))
                out[s][1].append(int(exl[j]))
        return out

    try:
        print(f"case: C4 full size, batch {B}, prompts {min(lens)}..{max(lens)}", flush=True)
        both = run(list(range(B)))
        picks = sorted({int(np.argmin(lens)), int(np.argmax(lens)), B // 2})
        s0 = picks[-1]
        # the cache of one sequence after the batch run + flush, against a full-depth prompt phase over its tokens
        cache.flush(list(range(B)))
        n_pos = lens[s0] + n_new - 1
        seq = np.concatenate([prompts[s0], np.array(both[s0][0][:-1], np.int32)])
        ee.prefill(gm, cache, B, seq, 1.0)
        for l in (0, 8, 16, 31):
            assert cache.filled(s0, l) == n_pos and cache.filled(B, l) == n_pos
            k0, v0 = cache.read(s0, l, lens[s0] - 8, n_new + 7)
            k1, v1 = cache.read(B, l, lens[s0] - 8, n_new + 7)
            kv_check(k0, k1, "bf16", "K", l), kv_check(v0, v1, "bf16", "V", l)
        cache.reset(B)
        for s in picks:
            print(f"case: C4 full size, sequence {s} alone (prompt {lens[s]})", flush=True)
            solo = run([s])
            assert solo[s] == both[s], (s, solo[s], both[s])
    finally:
        cache.close()
        gm.close()


def test_c5_full_size_invariants():
    """C5 as benchmarked (30B-shaped, 60 layers, 65 GB of weights, 4 sequences of 2048 prompt tokens): threshold 1 is
    repeatable bit for bit and never exits, threshold 0 exits at the first exit except on forced steps, and after a
    flush the cache of a sequence equals a full-depth prompt phase over what it generated."""
    wl = CONFIGS["C5"]
    shape, B, n_prompt, n_new = wl.shape, wl.batch, wl.prompt_len[0], 20
    prompts = [prompt_tokens(shape.vocab, n_prompt, wl.prompt_seed + b).numpy() for b in range(B)]
    gm = load_gpu_model(shape, wl.weight_seed, max_positions=n_prompt + n_new + 8, max_rows=min(256, 16 * B + 48), max_seqs=B)
    cache = ee.KvCache(gm, B + 1, (B + 1) * (n_prompt + n_new + 72), 64, 15)
    L, e1 = shape.n_layers, shape.exit_layers[0]
    ids = list(range(B))

    def run(tau):
        seqs = ee.Sequences(L)
        out = {s: ([], []) for s in ids}
        for s in ids:
            cache.reset(s)
            tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], tau)
            seqs.start(s, tok)
            out[s][0].append(int(tok))
            out[s][1].append(int(ex))
        for _ in range(n_new - 1):
            ro, tk, pm = seqs.rows(ids)
            nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
            seqs.update(ids, nt, exl)
            for j, s in enumerate(ids):
                out[s][0].append(int(nt[j]))
                out[s][1].append(int(exl[j]))
        return out

    try:
        print("case: C5 full size tau 1.0", flush=True)
        a = run(1.0)
        assert all(set(a[s][1]) == {L} for s in ids)
        assert run(1.0) == a, "two runs must be bit-identical (fixed-order reductions)"
        print("case: C5 full size tau 0.0", flush=True)
        z = run(0.0)
        for s in ids:
            x0 = z[s][1]
            assert x0[0] == e1 and all(x0[j] == (L if j % 16 == 0 else e1) for j in range(1, n_new)), x0
        print("case: C5 full size tau 0.5 + KV invariant", flush=True)
        h = run(wl.thresholds[0])
        cache.flush(ids)
        n_pos = n_prompt + n_new - 1
        seq = np.concatenate([prompts[1], np.array(h[1][0][:-1], np.int32)])
        ee.prefill(gm, cache, B, seq, 1.0)
        for l in (0, 14, 15, 30, 59):
            assert cache.filled(1, l) == n_pos and cache.filled(B, l) == n_pos
            k0, v0 = cache.read(1, l, n_prompt - 8, n_new + 7)
            k1, v1 = cache.read(B, l, n_prompt - 8, n_new + 7)
            kv_check(k0, k1, "bf16", "K", l), kv_check(v0, v1, "bf16", "V", l)
    finally:
        cache.close()
        gm.close()


@pytest.mark.parametrize("head_terms", [2, 1])
def test_c3_shape_prompt_phase_scored(head_terms):
    """Prompt phase through the GEMM path at the 7B widths (2 layers, exit after the first): cached K/V of every
    position and both heads scored on sampled positions against the oracle's cache-free forward; the scored heads
    on both terms of their input and on the leading one only (the library's default)."""
    from common import TOL_CONF_ONE_TERM, flip_guard
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,))
    n = 200
    O.set_threads(16)
    om, gm = build_pair(shape, 0, max_positions=256, scored_head_terms=head_terms)
    tol_pos = TOL_CONF["bf16"] if head_terms == 2 else TOL_CONF_ONE_TERM
    try:
        print(f"case: C3-shaped scored prompt phase, head terms {head_terms}", flush=True)
        p = prompt_tokens(shape.vocab, n, 5).numpy()
        cache = ee.KvCache(gm, 1, 256, 64, 15)
        tok, ex, conf, ptok, pconf = ee.prefill_scored(gm, cache, 0, p, 0.2)
        hid, ko, vo = om.forward_sequence(p)
        for l in range(2):
            k, v = cache.read(0, l, 0, n)
            kv_check(k, ko[l], "bf16", "K", l), kv_check(v, vo[l], "bf16", "V", l)
        assert rel_err(cache.read_hidden(0), hid[2][n - 1]) <= TOL
        forced = 0
        for hi, layer in enumerate((1, 2)):
            for pos in list(range(0, n, 9)) + list(range(n - 6, n)):
                _, dg = om.head_row(hi, hid[layer][pos])
                if int(ptok[hi, pos]) != dg["argmax"]:
                    assert dg["top1"] - dg["top2"] < flip_guard(dg, head_terms) and int(ptok[hi, pos]) == dg["arg2"], (hi, pos, dg)
                    forced += 1
                assert abs(float(pconf[hi, pos]) - dg["conf"]) <= tol_pos, (hi, pos, float(pconf[hi, pos]), dg["conf"])
        assert forced <= 3
        assert abs(float(conf[1]) - float(pconf[1, n - 1])) <= (1e-4 if head_terms == 2 else tol_pos)
        cache.close()
    finally:
        gm.close()
        O.set_threads(1)


def test_c3_shape_batch_many_rows_equals_solo():
    """7B widths, 2 layers, three ragged sequences at threshold 0: the deferred rows pile up to 3 x 16 = 48 rows per
    launch (packed row operands, several column tiles per workgroup, 2 and 4 row tiles); every sequence must emit
    exactly what it emits alone (the solo path is the one checked against the oracle above)."""
    shape = dataclasses.replace(CONFIGS["C3"].shape, n_layers=2, exit_layers=(1,))
    gm = load_gpu_model(shape, 0, max_positions=256, max_rows=64, max_seqs=4)
    n_new, tau, cap = 40, 0.0, 15
    prompts = [prompt_tokens(shape.vocab, 20 + 13 * s, 60 + s).numpy() for s in range(3)]
    ids = [0, 1, 2]

    def run(which):
        cache = ee.KvCache(gm, 4, 1024, 64, cap)
        seqs = ee.Sequences(shape.n_layers)
        out = {s: ([], []) for s in which}
        for s in which:
            tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], tau)
            seqs.start(s, tok)
            out[s][0].append(tok)
            out[s][1].append(ex)
        max_rows = 0
        for _ in range(n_new - 1):
            ro, tk, pm = seqs.rows(which)
            max_rows = max(max_rows, len(tk))
            nt, exl, _ = ee.decode_step(gm, cache, which, ro, tk, pm, tau)
            seqs.update(which, nt, exl)
            for j, s in enumerate(which):
                out[s][0].append(int(nt[j]))
                out[s][1].append(int(exl[j]))
        cache.flush(which)
        kv = {s: cache.read(s, 1, 0, len(prompts[s]) + n_new - 1) for s in which}
        cache.close()
        return out, max_rows, kv

    try:
        print("case: C3-shaped batch of many rows", flush=True)
        both, max_rows, kvb = run(ids)
        assert max_rows > 32
        for s in ids:
            solo, _, kvs = run([s])
            assert both[s][0] == solo[s][0] and both[s][1] == solo[s][1], s
            kv_check(kvb[s][0], kvs[s][0], "bf16", "K", 1), kv_check(kvb[s][1], kvs[s][1], "bf16", "V", 1)
    finally:
        gm.close()
