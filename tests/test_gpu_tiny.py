"""GPU parity on the tiny workload (C1, fp32) and on a tiny bf16 model, through the C ABI, against the
CPU oracle: tokens and exit layers exact outside the guard band, hidden states / logits / cached KV
within the stated relative error (1e-4 for fp32, 2e-3 for bf16)."""
import os
import tempfile

import numpy as np
import pytest
import torch

import paper_2312_04916_amd as ee
from oracle import oracle as O
from oracle.from_workload import build_model
from workload import CONFIGS, ModelShape, prompt_tokens, write_weight_file

from common import TOL, TOL_CONF, ee_config_of, kv_check, load_gpu_model, lockstep, rel_err

pytestmark = pytest.mark.gpu

C1 = CONFIGS["C1"]
TINY_BF16 = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "bf16", 0.02, 0.3)


@pytest.fixture(scope="module", params=["f32", "bf16"])
def pair(request):
    shape = C1.shape if request.param == "f32" else TINY_BF16
    om = build_model(shape, 0, gain_jitter=0.1)
    gm = load_gpu_model(shape, 0, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=2)
    yield shape, om, gm
    gm.close()


@pytest.fixture(scope="module")
def prompt():
    return prompt_tokens(C1.shape.vocab, C1.prompt_len[0], C1.prompt_seed).numpy()


def new_cache(gm, max_pending=40, block_tokens=32, max_seqs=2):
    return ee.KvCache(gm, max_seqs, 512, block_tokens, max_pending)


@pytest.mark.parametrize("tau", [0.0, 0.2, 0.35, 0.5, 0.8, 1.0])
def test_lockstep_generation(pair, prompt, tau):
    shape, om, gm = pair
    print(f"case: lockstep {shape.dtype} tau={tau}", flush=True)
    cache = new_cache(gm)
    logits = gm.enable_logits(1)
    rep = lockstep(gm, cache, om, prompt, C1.new_tokens, tau, max_pending=40, logits=logits)
    assert not rep.mismatches, rep.mismatches[:5]
    tol = TOL[shape.dtype]
    assert rep.max_hidden_err <= tol, rep.max_hidden_err
    assert rep.max_logit_err <= tol, rep.max_logit_err
    assert rep.max_conf_err <= TOL_CONF[shape.dtype]
    if tau == 0.0:
        assert set(rep.exit_layers) == {shape.exit_layers[0]}
    if tau == 1.0:
        assert set(rep.exit_layers) == {shape.n_layers}
        if rep.teacher_forced == 0:
            assert rep.tokens == om.generate_plain(prompt, C1.new_tokens).tolist()
    if shape.dtype == "f32":
        assert rep.teacher_forced == 0
        toks, exits = om.generate_g0(prompt, C1.new_tokens, tau)
        assert rep.tokens == toks.tolist() and rep.exit_layers == exits.tolist()
    # KV recomputation: after a flush the cache equals the oracle's (which equals a full-depth forward)
    n_pos = len(prompt) + C1.new_tokens - 1
    st = rep.state
    cache.flush([0])
    st.flush()
    assert cache.pending(0) == 0
    for l in range(shape.n_layers):
        assert cache.filled(0, l) == n_pos
        k, v = cache.read(0, l, 0, n_pos)
        ko, vo = st.kv_read(l, 0, n_pos)
        kv_check(k, ko, shape.dtype, "K", l), kv_check(v, vo, shape.dtype, "V", l)
    gm.enable_logits(1)
    cache.close()


def test_kv_is_incomplete_before_flush_and_watermarks(pair, prompt):
    shape, om, gm = pair
    print(f"case: watermarks {shape.dtype}", flush=True)
    cache = new_cache(gm)
    rep = lockstep(gm, cache, om, prompt, 9, 0.0, max_pending=40, check_hidden=False)
    P = len(prompt)
    assert cache.pending(0) == 8
    assert cache.filled(0, 0) == P + 8 and cache.filled(0, 1) == P and cache.filled(0, 3) == P
    cache.close()


@pytest.mark.parametrize("cap", [1, 3])
def test_forced_full_depth(pair, prompt, cap):
    shape, om, gm = pair
    print(f"case: cap {shape.dtype} cap={cap}", flush=True)
    cache = new_cache(gm, max_pending=cap)
    rep = lockstep(gm, cache, om, prompt, 14, 0.0, max_pending=cap)
    assert not rep.mismatches, rep.mismatches[:5]
    L, e1 = shape.n_layers, shape.exit_layers[0]
    for j in range(1, 14):
        assert rep.exit_layers[j] == (L if j % (cap + 1) == 0 else e1)
    assert rep.forced_full == (14 - 1) // (cap + 1)
    cache.close()


@pytest.mark.parametrize("tau,cap", [(0.0, 3), (0.35, 40), (0.2, 6)])
def test_refeed_mode_matches_oracle_and_resume_mode(pair, prompt, tau, cap):
    """Deferred tokens fed again from the embedding (the paper's literal wording, which is what the oracle's G1 does)
    give the same tokens, exit layers and KV as resuming them from their saved residual rows."""
    shape, om, gm = pair
    print(f"case: refeed {shape.dtype} tau={tau} cap={cap}", flush=True)
    outs = []
    for refeed in (False, True):
        cache = new_cache(gm, max_pending=cap)
        cache.set_refeed(refeed)
        rep = lockstep(gm, cache, om, prompt, 26, tau, max_pending=cap)
        assert not rep.mismatches, rep.mismatches[:5]
        assert rep.max_hidden_err <= TOL[shape.dtype]
        n_pos = len(prompt) + 25
        cache.flush([0])
        assert cache.pending(0) == 0
        kv = [cache.read(0, l, 0, n_pos) for l in range(shape.n_layers)]
        outs.append((rep.tokens, rep.exit_layers, kv))
        rep.state.flush()
        for l in range(shape.n_layers):
            ko, vo = rep.state.kv_read(l, 0, n_pos)
            kv_check(kv[l][0], ko, shape.dtype, "K", l), kv_check(kv[l][1], vo, shape.dtype, "V", l)
        cache.close()
    assert outs[0][0] == outs[1][0] and outs[0][1] == outs[1][1]
    for l in range(shape.n_layers):
        kv_check(outs[1][2][l][0], outs[0][2][l][0], shape.dtype, "K", l), kv_check(outs[1][2][l][1], outs[0][2][l][1], shape.dtype, "V", l)


def test_cap_one_alternates_and_cap_63_fills_a_whole_pass(pair, prompt):
    """Degenerate caps: with max_pending 1 and threshold 0 every second step is forced to full depth; with a cap of 63
    and threshold 0 one sequence piles up 64 rows (the model's max_rows here) before the forced step."""
    shape, om, gm = pair
    print(f"case: caps 1 / 63 {shape.dtype}", flush=True)
    def decode(cap, tau_decode):
        cache = new_cache(gm, max_pending=cap)
        tok, ex, _ = ee.prefill(gm, cache, 0, prompt, 0.0)
        seqs = ee.Sequences(shape.n_layers)
        seqs.start(0, tok)
        toks, exits = [tok], [ex]
        for _ in range(11):
            ro, tk, pm = seqs.rows([0])
            nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, tau_decode)
            seqs.update([0], nt, exl)
            toks.append(int(nt[0]))
            exits.append(int(exl[0]))
        cache.flush([0])
        assert cache.pending(0) == 0
        cache.close()
        return toks, exits

    _, alt_exits = decode(1, 0.0)
    assert alt_exits[1:] == [shape.exit_layers[0], shape.n_layers] * 5 + [shape.exit_layers[0]]
    cache = ee.KvCache(gm, 1, 512, 32, 63)
    rep = lockstep(gm, cache, om, prompt, 70, 0.0, max_pending=63, max_positions=128)
    assert not rep.mismatches, rep.mismatches[:5]
    assert rep.exit_layers[64] == shape.n_layers and rep.forced_full == 1 and cache.pending(0) == 5
    assert rep.max_hidden_err <= TOL[shape.dtype]
    cache.close()


def test_no_cap_never_forces_and_overflow_is_refused_without_side_effects(pair, prompt):
    """max_pending <= 0 is "no cap" on both sides of the boundary: at threshold 0 every token leaves at the first exit
    and no step is forced; once the rows of a step would exceed the model's max_rows (64 here) the step is refused
    with EE_ERR_NOMEM and nothing has changed: after a flush the same call goes through."""
    shape, om, gm = pair
    print(f"case: no cap {shape.dtype}", flush=True)
    cache = ee.KvCache(gm, 1, 512, 32, 0)
    rep = lockstep(gm, cache, om, prompt, 64, 0.0, max_pending=0, max_positions=128)
    assert not rep.mismatches, rep.mismatches[:5]
    assert set(rep.exit_layers) == {shape.exit_layers[0]} and rep.forced_full == 0
    assert cache.pending(0) == 63 and rep.max_hidden_err <= TOL[shape.dtype]
    seqs = rep.seqs
    ro, tk, pm = seqs.rows([0])       # 63 deferred rows + the current one: exactly max_rows
    nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, 0.0)
    seqs.update([0], nt, exl)
    ro, tk, pm = seqs.rows([0])       # 65 rows: one too many
    filled = [cache.filled(0, l) for l in range(shape.n_layers)]
    with pytest.raises(ee.EeError) as e:
        ee.decode_step(gm, cache, [0], ro, tk, pm, 0.0)
    assert e.value.code == -2
    assert cache.pending(0) == 64 and [cache.filled(0, l) for l in range(shape.n_layers)] == filled
    cache.flush([0])
    assert cache.pending(0) == 0
    seqs.pending[0] = []
    ro, tk, pm = seqs.rows([0])
    nt2, exl2, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, 0.0)
    # the oracle, flushed at the same point, emits the same token
    st = rep.state
    t_o, x_o, _ = st.decode_step(rep.tokens[-1], 0.0)
    assert (t_o, x_o) == (int(nt[0]), int(exl[0]))
    st.flush()
    t_o, x_o, _ = st.decode_step(int(nt[0]), 0.0)
    assert (t_o, x_o) == (int(nt2[0]), int(exl2[0]))
    cache.close()


def test_refeed_mode_cannot_change_while_tokens_are_deferred(pair, prompt):
    """With tokens on the deferred list the saved residual rows belong to the mode that wrote them: the switch is
    refused (EE_ERR_STATE) until a flush or a full-depth step has emptied the list, and generation that switches at
    such a point matches the oracle throughout."""
    shape, om, gm = pair
    print(f"case: refeed switch {shape.dtype}", flush=True)
    cache = new_cache(gm, max_pending=6)
    cache.set_refeed(True)
    rep = lockstep(gm, cache, om, prompt, 6, 0.0, max_pending=6, max_positions=64)
    assert not rep.mismatches and cache.pending(0) == 5
    with pytest.raises(ee.EeError) as e:
        cache.set_refeed(False)
    assert e.value.code == -4
    cache.set_refeed(True)            # setting the mode it already has is fine
    cache.flush([0])
    rep.state.flush()
    cache.set_refeed(False)
    seqs, st = rep.seqs, rep.state
    seqs.pending[0] = []
    tok = rep.tokens[-1]
    for _ in range(5):
        ro, tk, pm = seqs.rows([0])
        nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, 0.0)
        seqs.update([0], nt, exl)
        t_o, x_o, _ = st.decode_step(tok, 0.0)
        assert (t_o, x_o) == (int(nt[0]), int(exl[0]))
        tok = t_o
    n_pos = len(prompt) + 10
    cache.flush([0])
    st.flush()
    for l in range(shape.n_layers):
        k, v = cache.read(0, l, 0, n_pos)
        ko, vo = st.kv_read(l, 0, n_pos)
        kv_check(k, ko, shape.dtype, "K", l), kv_check(v, vo, shape.dtype, "V", l)
    cache.close()


def test_two_sequences_equal_each_alone(pair, prompt):
    """Sequences are independent: a batch of two ragged sequences gives what each gives alone."""
    shape, om, gm = pair
    print(f"case: batch2 {shape.dtype}", flush=True)
    tau, n_new = 0.35, 20
    p2 = prompt_tokens(shape.vocab, 23, 7).numpy()
    alone = []
    for p in (prompt, p2):
        cache = new_cache(gm)
        rep = lockstep(gm, cache, om, p, n_new, tau, max_pending=40, check_hidden=False)
        alone.append((rep.tokens, rep.exit_layers))
        cache.close()
    cache = new_cache(gm)
    seqs = ee.Sequences(shape.n_layers)
    out = {0: ([], []), 1: ([], [])}
    for s, p in ((0, prompt), (1, p2)):
        tok, ex, _ = ee.prefill(gm, cache, s, p, tau)
        seqs.start(s, tok)
        out[s][0].append(tok)
        out[s][1].append(ex)
    for _ in range(n_new - 1):
        ro, tk, pm = seqs.rows([0, 1])
        nt, exl, _ = ee.decode_step(gm, cache, [0, 1], ro, tk, pm, tau)
        seqs.update([0, 1], nt, exl)
        for s in (0, 1):
            out[s][0].append(int(nt[s]))
            out[s][1].append(int(exl[s]))
    for s in (0, 1):
        assert out[s][0] == alone[s][0] and out[s][1] == alone[s][1]
    cache.close()


def test_long_prompt_spans_chunks_and_blocks(pair):
    """Prompt longer than one prefill chunk (64 rows) and several cache blocks, ragged tail."""
    shape, om, gm = pair
    print(f"case: long prompt {shape.dtype}", flush=True)
    p = prompt_tokens(shape.vocab, 150, 11).numpy()
    cache = new_cache(gm, max_pending=5)
    rep = lockstep(gm, cache, om, p, 12, 0.35, max_pending=5)
    assert not rep.mismatches, rep.mismatches[:5]
    assert rep.max_hidden_err <= TOL[shape.dtype]
    k, v = cache.read(0, shape.n_layers - 1, 0, 150)
    ko, vo = rep.state.kv_read(shape.n_layers - 1, 0, 150)
    kv_check(k, ko, shape.dtype, "K", shape.n_layers - 1), kv_check(v, vo, shape.dtype, "V", shape.n_layers - 1)
    cache.close()


def test_model_load_from_file_matches_set_tensor(prompt):
    print("case: model_load file", flush=True)
    shape = C1.shape
    om = build_model(shape, 0)
    with tempfile.TemporaryDirectory() as td:
        path = os.path.join(td, "c1.eewt")
        write_weight_file(path, shape, 0, max_positions=256)
        gm = ee.model_load(ee_config_of(shape, 256), path, 64, 1)
    cache = ee.KvCache(gm, 1, 256, 32, 40)
    rep = lockstep(gm, cache, om, prompt, 12, 0.5, max_pending=40)
    assert not rep.mismatches and rep.max_hidden_err <= 1e-4
    cache.close()
    gm.close()


def test_error_codes(pair, prompt):
    shape, om, gm = pair
    print(f"case: errors {shape.dtype}", flush=True)
    cache = new_cache(gm, max_pending=4)

    def code(fn):
        with pytest.raises(ee.EeError) as e:
            fn()
        return e.value.code

    # decode before prefill; bad token; bad sequence id
    assert code(lambda: ee.decode_step(gm, cache, [0], [0, 1], [5], [0], 0.5)) == -4
    assert code(lambda: ee.prefill(gm, cache, 0, [shape.vocab], 0.5)) == -3
    assert code(lambda: ee.prefill(gm, cache, 9, [1, 2], 0.5)) == -3
    tok, ex, _ = ee.prefill(gm, cache, 0, prompt, 0.0)
    assert code(lambda: ee.prefill(gm, cache, 0, prompt, 0.0)) == -4          # sequence not empty
    nt, exl, _ = ee.decode_step(gm, cache, [0], [0, 1], [tok], [0], 0.0)      # exits early -> one pending
    assert cache.pending(0) == 1
    assert code(lambda: ee.decode_step(gm, cache, [0], [0, 1], [int(nt[0])], [0], 0.0)) == -4   # pending row missing
    assert code(lambda: ee.decode_step(gm, cache, [0], [0, 2], [tok + 1, int(nt[0])], [1, 0], 0.0)) == -4  # wrong id
    assert code(lambda: ee.decode_step(gm, cache, [0], [0, 2], [tok, int(nt[0])], [0, 0], 0.0)) == -4      # wrong mask
    assert code(lambda: ee.decode_step(gm, cache, [0, 0], [0, 2, 4], [tok, int(nt[0])] * 2, [1, 0, 1, 0], 0.0)) == -7
    assert code(lambda: ee.decode_step(gm, cache, [0], [0, 2], [tok, shape.vocab], [1, 0], 0.0)) == -3
    ee.decode_step(gm, cache, [0], [0, 2], [tok, int(nt[0])], [1, 0], 0.0)    # the right call still works
    assert cache.pending(0) == 2
    cache.reset(0)
    assert cache.pending(0) == 0 and cache.filled(0, 0) == 0
    # pool exhaustion: 2 sequences * 32-token blocks, 40 tokens in all -> 2 + 2 blocks
    small = ee.KvCache(gm, 2, 40, 32, 4)
    ee.prefill(gm, small, 0, prompt_tokens(shape.vocab, 100, 3).numpy(), 1.0)
    assert code(lambda: ee.prefill(gm, small, 1, prompt_tokens(shape.vocab, 40, 3).numpy(), 1.0)) == -2
    small.close()
    cache.close()


@pytest.mark.parametrize("hd,d,H", [(128, 256, 2), (64, 256, 4)])
def test_other_head_dims_with_split_kv(hd, d, H, min_wgs=0):
    """head_dim 128 / 64 models (MFMA attention with several KV splits and a ragged last tile)."""
    print(f"case: head_dim {hd}", flush=True)
    shape = ModelShape(3, d, H, hd, 512, 2048, (1, 2), "bf16", 0.02, 0.3 / (d / 128) ** 0.5)
    om = build_model(shape, 3, gain_jitter=0.1)
    gm = load_gpu_model(shape, 3, gain_jitter=0.1, max_positions=512, max_rows=64, max_seqs=1, gemm_min_workgroups=min_wgs)
    p = prompt_tokens(shape.vocab, 333, 5).numpy()
    cache = ee.KvCache(gm, 1, 512, 64, 6)
    logits = gm.enable_logits(1)
    rep = lockstep(gm, cache, om, p, 24, 0.3, max_pending=6, logits=logits)
    assert not rep.mismatches, rep.mismatches[:5]
    assert rep.max_hidden_err <= TOL["bf16"] and rep.max_logit_err <= TOL["bf16"]
    assert len(set(rep.exit_layers)) >= 2
    n_pos = len(p) + 23
    cache.flush([0])
    rep.state.flush()
    for l in range(shape.n_layers):
        k, v = cache.read(0, l, 0, n_pos)
        ko, vo = rep.state.kv_read(l, 0, n_pos)
        kv_check(k, ko, "bf16", "K", l), kv_check(v, vo, "bf16", "V", l)
    print(f"head_dim {hd}: hidden err {rep.max_hidden_err:.2e} logit err {rep.max_logit_err:.2e} "
          f"teacher-forced {rep.teacher_forced} exits {sorted(set(rep.exit_layers))}", flush=True)
    cache.close()
    gm.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_maximum_rows_per_step(dtype):
    """Four sequences with the largest cap at threshold 0 reach 4 x 64 = 256 rows in one launch (the library's
    maximum, four row passes); each must emit what it emits alone, and one row more is refused."""
    print(f"case: 256 rows {dtype}", flush=True)
    shape = C1.shape if dtype == "f32" else TINY_BF16
    gm = load_gpu_model(shape, 0, gain_jitter=0.1, max_positions=256, max_rows=256, max_seqs=5)
    n_new, cap = 66, 63
    prompts = [prompt_tokens(shape.vocab, 5 + 3 * s, 70 + s).numpy() for s in range(5)]

    def run(which, expect_fail_at=None):
        cache = ee.KvCache(gm, 5, 2048, 32, cap)
        seqs = ee.Sequences(shape.n_layers)
        out = {s: [] for s in which}
        for s in which:
            tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], 0.0)
            seqs.start(s, tok)
            out[s].append((tok, ex))
        max_rows = 0
        for step in range(n_new - 1):
            ro, tk, pm = seqs.rows(which)
            max_rows = max(max_rows, len(tk))
            if expect_fail_at is not None and len(tk) > 256:
                with pytest.raises(ee.EeError) as e:
                    ee.decode_step(gm, cache, which, ro, tk, pm, 0.0)
                assert e.value.code == -2
                cache.close()
                return None, max_rows
            nt, exl, _ = ee.decode_step(gm, cache, which, ro, tk, pm, 0.0)
            seqs.update(which, nt, exl)
            for j, s in enumerate(which):
                out[s].append((int(nt[j]), int(exl[j])))
        cache.close()
        return out, max_rows

    both, max_rows = run([0, 1, 2, 3])
    assert max_rows == 256
    for s in range(4):
        solo, _ = run([s])
        assert both[s] == solo[s], s
    _, max_rows = run([0, 1, 2, 3, 4], expect_fail_at=True)   # five sequences would need 257+ rows: refused
    assert max_rows > 256
    gm.close()


def test_workload_generator_is_device_independent():
    """The seeded generator must give the same bits on the CPU (oracle side) and on the GPU (library side)."""
    from workload import TensorKind, model_tensor
    for shape in (C1.shape, TINY_BF16):
        for kind in (TensorKind.EMBED, TensorKind.WG, TensorKind.EXIT_HEAD, TensorKind.ATTN_NORM):
            a = model_tensor(shape, kind, 1 if kind != TensorKind.EMBED else 0, 5, "cpu", 0.1)
            b = model_tensor(shape, kind, 1 if kind != TensorKind.EMBED else 0, 5, "cuda:0", 0.1).cpu()
            assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                               b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))
    assert torch.equal(prompt_tokens(50304, 1000, 3, "cpu"), prompt_tokens(50304, 1000, 3, "cuda:0").cpu())


def test_ragged_batch_with_several_tiles_per_workgroup():
    """The same ragged batch with the GEMMs forced to give every workgroup several column tiles (the variants that
    the 7B shapes take when a step has many rows), including a head over more rows than LDS holds."""
    for min_wgs in (1, 16):  # 1: two or four tiles; 16: as many tiles as there would be rounds of 8 workgroups (3..6)
        test_ragged_batch_with_more_than_64_rows("bf16", min_wgs)
        test_other_head_dims_with_split_kv(64, 256, 4, min_wgs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_batch_with_more_than_64_rows(dtype, min_wgs=0):
    """Six ragged sequences at threshold 0.0 pile up deferred rows (up to 6 x 16 = 96 rows in one launch, more
    than one 64-row pass); every sequence must give exactly what it gives alone, and one is checked in
    lockstep against the oracle."""
    print(f"case: ragged batch {dtype}", flush=True)
    shape = C1.shape if dtype == "f32" else TINY_BF16
    om = build_model(shape, 0, gain_jitter=0.1)
    gm = load_gpu_model(shape, 0, gain_jitter=0.1, max_positions=256, max_rows=128, max_seqs=8, gemm_min_workgroups=min_wgs)
    n_seq, n_new, tau, cap = 6, 36, 0.0, 15
    prompts = [prompt_tokens(shape.vocab, 9 + 7 * s, 20 + s).numpy() for s in range(n_seq)]
    solo = []
    for s in range(n_seq):
        cache = ee.KvCache(gm, 8, 2048, 32, cap)
        rep = lockstep(gm, cache, om, prompts[s], n_new, tau, max_pending=cap, check_hidden=(s == 0))
        if s == 0:
            assert not rep.mismatches and rep.max_hidden_err <= TOL[dtype]
        solo.append((rep.tokens, rep.exit_layers))
        cache.close()
    cache = ee.KvCache(gm, 8, 2048, 32, cap)
    seqs = ee.Sequences(shape.n_layers)
    out = [([], []) for _ in range(n_seq)]
    ids = list(range(n_seq))
    for s in ids:
        tok, ex, _ = ee.prefill(gm, cache, s, prompts[s], tau)
        seqs.start(s, tok)
        out[s][0].append(tok)
        out[s][1].append(ex)
    max_rows = 0
    for _ in range(n_new - 1):
        ro, tk, pm = seqs.rows(ids)
        max_rows = max(max_rows, len(tk))
        nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
        seqs.update(ids, nt, exl)
        for s in ids:
            out[s][0].append(int(nt[s]))
            out[s][1].append(int(exl[s]))
    assert max_rows > 64
    for s in ids:
        assert out[s][0] == solo[s][0] and out[s][1] == solo[s][1], s
    cache.flush(ids)
    assert all(cache.pending(s) == 0 for s in ids)
    cache.close()
    gm.close()


def test_measurement_hook_counts_and_samples_launches():
    """ee_profile_begin / ee_profile_every / ee_profile_end: every launch of the chosen kernel family carries an event
    pair, or every n-th one; the counts follow from the number of layers and steps, the durations are positive, and
    the tokens are those of an unmeasured run."""
    print("case: measurement hook", flush=True)
    shape = TINY_BF16
    gm = load_gpu_model(shape, 0, gain_jitter=0.1, max_positions=64, max_rows=16, max_seqs=1)
    prompt = prompt_tokens(shape.vocab, 9, 2).numpy()

    def run(kernel=None, every=1):
        cache = ee.KvCache(gm, 1, 64, 32, 4)
        seqs = ee.Sequences(shape.n_layers)
        tok, _, _ = ee.prefill(gm, cache, 0, prompt, 1.0)
        seqs.start(0, tok)
        toks = [int(tok)]
        if kernel is not None:
            gm.profile_begin(kernel, max_launches=256, every=every)
        for _ in range(6):
            ro, tk, pm = seqs.rows([0])
            nt, exl, _ = ee.decode_step(gm, cache, [0], ro, tk, pm, 1.0)
            seqs.update([0], nt, exl)
            toks.append(int(nt[0]))
        prof = gm.profile_end() if kernel is not None else None
        cache.close()
        return toks, prof

    ref, _ = run()
    launches = 6 * shape.n_layers  # one gate|up launch per layer and step at full depth
    for every in (1, 4, 5):
        toks, (n, ms) = run(ee.EE_K_SWIGLU, every)
        assert toks == ref
        assert n == (launches + every - 1) // every, (every, n)
        assert ms > 0.0
    toks, (n, ms) = run(ee.EE_K_HEAD)  # the final head, once per step
    assert toks == ref and n == 6 and ms > 0.0
    gm.close()


def test_lane_reductions_equal_the_shuffle_butterflies():
    """The wave-wide and four-row reductions the kernels use (lane swaps, row rotates) against the xor butterflies over
    shuffles that they stand for: a million pseudo-random values, every result compared bit for bit on the device."""
    gm = load_gpu_model(TINY_BF16, 0, max_positions=64, max_rows=16, max_seqs=1)
    try:
        assert gm.lane_reduction_mismatches() == 0
    finally:
        gm.close()
