"""Pins of the oracle's generators: the plain definition G0, the KV-recomputation mechanism G1, the
forced full-depth rule, and the statements of the paper that fix behaviour (Section 5.2: threshold 1
disables exits; Appendix B.1: the output does not depend on the inference method; Section 4: after
recomputation no KV entry is missing).  CPU only.
"""
import json
import os

import numpy as np
import pytest
import scipy.special

from oracle import oracle as O
from oracle.from_workload import build_model
from workload import CONFIGS, ModelShape, TensorKind, prompt_tokens

C1 = CONFIGS["C1"]
N_NEW = C1.new_tokens
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "c1_generation.json")


@pytest.fixture(scope="module")
def model():
    return build_model(C1.shape, C1.weight_seed, gain_jitter=0.1)


@pytest.fixture(scope="module")
def prompt():
    return prompt_tokens(C1.shape.vocab, C1.prompt_len[0], C1.prompt_seed).numpy()


def pick(diags, tau):
    """The exit rule on a list of head evaluations in depth order (last = final head)."""
    if tau < 1.0:
        for d in diags[:-1]:
            if d["conf"] >= tau:
                return d["argmax"], d["layer"]
    return diags[-1]["argmax"], diags[-1]["layer"]


def run_g1(model, prompt, n_new, tau, max_pending=0, max_pos=128):
    st = O.State(model, max_pos, max_pending)
    tok, ex = pick(st.prefill(prompt), tau)
    toks, exits, pend = [tok], [ex], [st.n_pending()]
    for _ in range(n_new - 1):
        tok, ex, _ = st.decode_step(tok, tau)
        toks.append(tok)
        exits.append(ex)
        pend.append(st.n_pending())
        f = [st.filled(s) for s in range(model.cfg.n_exits + 1)]
        assert all(f[i] >= f[i + 1] for i in range(len(f) - 1)), "watermarks must be non-increasing in depth"
    return st, np.array(toks), np.array(exits), pend


@pytest.mark.parametrize("tau", [0.0, 0.2, 0.35, 0.5, 0.8, 1.0])
def test_g1_equals_g0_bit_exact(model, prompt, tau):
    t0, e0 = model.generate_g0(prompt, N_NEW, tau)
    _, t1, e1, _ = run_g1(model, prompt, N_NEW, tau)
    assert np.array_equal(t0, t1) and np.array_equal(e0, e1)


def test_exit_mix_is_not_degenerate(model, prompt):
    # at least one threshold must exercise all three depths, or the G1 == G0 pin proves little
    seen = set()
    for tau in (0.2, 0.35, 0.5):
        _, e0 = model.generate_g0(prompt, N_NEW, tau)
        seen |= set(e0.tolist())
    assert seen == {1, 2, 4}


def test_threshold_one_is_plain_greedy(model, prompt):
    t0, e0 = model.generate_g0(prompt, N_NEW, 1.0)
    assert np.array_equal(t0, model.generate_plain(prompt, N_NEW))
    assert set(e0.tolist()) == {C1.shape.n_layers}
    _, t1, e1, pend = run_g1(model, prompt, N_NEW, 1.0)
    assert np.array_equal(t1, t0) and max(pend) == 0


def test_threshold_zero_exits_at_first_exit(model, prompt):
    _, t1, e1, pend = run_g1(model, prompt, N_NEW, 0.0)
    assert set(e1.tolist()) == {C1.shape.exit_layers[0]}
    assert pend == list(range(0, N_NEW))  # nothing ever clears the list without a cap


@pytest.mark.parametrize("tau", [0.0, 0.35])
def test_kv_after_flush_equals_full_depth_forward(model, prompt, tau):
    st, toks, exits, _ = run_g1(model, prompt, N_NEW, tau)
    n_pos = len(prompt) + N_NEW - 1  # the last emitted token is never an input
    assert st.filled(0) == n_pos
    had_pending = st.n_pending()
    st.flush()
    assert st.n_pending() == 0 and all(st.filled(s) == n_pos for s in range(3))
    seq = np.concatenate([prompt, toks[:-1]]).astype(np.int32)
    _, k_ref, v_ref = model.forward_sequence(seq)
    for l in range(C1.shape.n_layers):
        k, v = st.kv_read(l, 0, n_pos)
        assert np.array_equal(k, k_ref[l]) and np.array_equal(v, v_ref[l])
    if tau == 0.0:
        assert had_pending == N_NEW - 1


def test_kv_is_missing_before_flush(model, prompt):
    st, toks, _, _ = run_g1(model, prompt, 8, 0.0)
    n_pos = len(prompt) + 7
    seq = np.concatenate([prompt, toks[:-1]]).astype(np.int32)
    _, k_ref, _ = model.forward_sequence(seq)
    k_shallow, _ = st.kv_read(0, 0, n_pos)
    k_deep, _ = st.kv_read(3, 0, n_pos)
    assert np.array_equal(k_shallow, k_ref[0])
    assert np.array_equal(k_deep[:len(prompt)], k_ref[3][:len(prompt)])
    assert not np.array_equal(k_deep[len(prompt):], k_ref[3][len(prompt):])
    assert st.filled(0) == n_pos and st.filled(2) == len(prompt)


@pytest.mark.parametrize("cap", [1, 3])
def test_forced_full_depth_when_pending_reaches_cap(model, prompt, cap):
    st, t1, e1, pend = run_g1(model, prompt, N_NEW, 0.0, max_pending=cap)
    assert max(pend) <= cap
    L, e_first = C1.shape.n_layers, C1.shape.exit_layers[0]
    # token 0 comes from prefill; then `cap` early exits, then one forced full step, repeating
    for j in range(1, N_NEW):
        assert e1[j] == (L if j % (cap + 1) == 0 else e_first)
    t0, e0 = model.generate_g0(prompt, N_NEW, 0.0, max_pending=cap)
    assert np.array_equal(t0, t1) and np.array_equal(e0, e1)


@pytest.mark.parametrize("tau", [0.35, 0.5])
def test_every_emitted_token_obeys_the_rule(model, prompt, tau):
    """Teacher-forced re-check with the cache-free forward: confidence below tau at every earlier
    exit, at or above it at the exit taken, and the token is the arg max there."""
    toks, exits = model.generate_g0(prompt, N_NEW, tau)
    sh = C1.shape
    seq = list(prompt)
    for j in range(N_NEW):
        hid, _, _ = model.forward_sequence(np.array(seq, np.int32))
        for i, e in enumerate(sh.exit_layers):
            _, d = model.head_row(i, np.ascontiguousarray(hid[e, -1]))
            if e < exits[j]:
                assert d["conf"] < tau
            elif e == exits[j]:
                assert d["conf"] >= tau and d["argmax"] == toks[j]
        if exits[j] == sh.n_layers:
            _, d = model.head_row(len(sh.exit_layers), np.ascontiguousarray(hid[sh.n_layers, -1]))
            assert d["argmax"] == toks[j]
        seq.append(int(toks[j]))


def test_step_parts_allow_teacher_forcing(model, prompt):
    """begin/advance/commit can end a step at an exit the rule would not take, with a chosen token."""
    st = O.State(model, 64, 0)
    tok, _ = pick(st.prefill(prompt), 1.0)
    assert st.step_begin(tok) is False
    depth, d = st.step_advance(True)
    assert depth == C1.shape.exit_layers[0] and d["layer"] == depth
    st.step_commit(7)
    assert st.n_pending() == 1 and st.filled(0) == len(prompt) + 1 and st.filled(1) == len(prompt)
    assert st.step_begin(7) is False
    depth, d = st.step_advance(False)
    assert d is None
    depth, d = st.step_advance(False)
    depth, d = st.step_advance(False)
    assert depth == C1.shape.n_layers and d["layer"] == depth
    st.step_commit(d["argmax"])
    assert st.n_pending() == 0


# ---------------------------------------------------------------- whole forward against numpy fp64

def numpy_forward(shape: ModelShape, model: O.Model, tokens):
    """An fp64 forward of the whole sequence at once (matrix form, causal mask) from library routines."""
    T = lambda kind, i=0: model.tensor(kind, i).astype(np.float64)
    n, d, H, hd = len(tokens), shape.d_model, shape.n_heads, shape.head_dim

    def rms(x, g):
        return g * x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + shape.rms_eps)

    def rope(x):  # x: [n][H][hd]
        half = hd // 2
        inv = shape.rope_base ** (-2.0 * np.arange(half) / hd)
        ang = np.arange(n)[:, None] * inv[None, :]
        c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        a, b = x[..., :half], x[..., half:]
        return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)

    x = T(TensorKind.EMBED)[np.asarray(tokens)]
    hidden = [x.copy()]
    mask = np.triu(np.full((n, n), -np.inf), k=1)
    for l in range(shape.n_layers):
        h = rms(x, T(TensorKind.ATTN_NORM, l))
        q = rope((h @ T(TensorKind.WQ, l).T).reshape(n, H, hd))
        k = rope((h @ T(TensorKind.WK, l).T).reshape(n, H, hd))
        v = (h @ T(TensorKind.WV, l).T).reshape(n, H, hd)
        s = np.einsum("ihc,jhc->hij", q, k) / np.sqrt(hd) + mask[None]
        a = np.einsum("hij,jhc->ihc", scipy.special.softmax(s, axis=-1), v).reshape(n, d)
        x = x + a @ T(TensorKind.WO, l).T
        h = rms(x, T(TensorKind.MLP_NORM, l))
        gate = h @ T(TensorKind.WG, l).T
        x = x + (gate * scipy.special.expit(gate) * (h @ T(TensorKind.WU, l).T)) @ T(TensorKind.WD, l).T
        hidden.append(x.copy())
    return np.stack(hidden)


def test_forward_sequence_matches_numpy_fp64(model, prompt):
    hid, _, _ = model.forward_sequence(prompt)
    ref = numpy_forward(C1.shape, model, prompt)
    for l in range(C1.shape.n_layers + 1):
        assert np.max(np.abs(hid[l] - ref[l])) <= 1e-5 * np.max(np.abs(ref[l]))
    # logits and confidence of every head on the last position
    for i in range(3):
        z, d = model.head_row(i, np.ascontiguousarray(hid[[1, 2, 4][i], -1]))
        gk, wk = ((TensorKind.EXIT_NORM, TensorKind.EXIT_HEAD) if i < 2 else
                  (TensorKind.FINAL_NORM, TensorKind.FINAL_HEAD))
        x = ref[[1, 2, 4][i], -1]
        h = model.tensor(gk, i if i < 2 else 0) * x / np.sqrt(np.mean(x * x) + C1.shape.rms_eps)
        zr = model.tensor(wk, i if i < 2 else 0).astype(np.float64) @ h
        assert np.max(np.abs(z - zr)) <= 1e-5 * np.max(np.abs(zr))
        assert np.isclose(d["conf"], scipy.special.softmax(zr).max(), rtol=1e-4)


# ---------------------------------------------------------------- bf16 storage mode

@pytest.fixture(scope="module")
def bf16_model():
    sh = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "bf16", 0.02, 0.3)
    return sh, build_model(sh, 0, gain_jitter=0.1)


@pytest.mark.parametrize("tau", [0.0, 0.35, 1.0])
def test_bf16_g1_equals_g0(bf16_model, prompt, tau):
    sh, m = bf16_model
    t0, e0 = m.generate_g0(prompt, 16, tau)
    _, t1, e1, _ = run_g1(m, prompt, 16, tau)
    assert np.array_equal(t0, t1) and np.array_equal(e0, e1)


def test_bf16_mode_is_close_to_fp32_and_cache_holds_bf16(bf16_model, model, prompt):
    sh, m = bf16_model
    hid_b, k_b, v_b = m.forward_sequence(prompt)
    # fp64 forward over the same bf16-rounded weights, no rounding of activations
    ref = numpy_forward(sh, _widened(m), prompt)
    for l in range(sh.n_layers + 1):
        assert np.max(np.abs(hid_b[l] - ref[l])) <= 2e-2 * np.max(np.abs(ref[l]))
    as_bf16 = np.vectorize(O.bf16_round)
    assert np.array_equal(k_b, as_bf16(k_b).astype(np.float32))
    assert np.array_equal(v_b, as_bf16(v_b).astype(np.float32))


class _widened:
    """View of a bf16 oracle model whose tensors read back as fp32 values."""

    def __init__(self, m):
        self.m = m

    def tensor(self, kind, i=0):
        a = self.m.tensor(kind, i)
        if a.dtype == np.uint16:
            return (a.astype(np.uint32) << 16).view(np.float32)
        return a


# ---------------------------------------------------------------- stored expected values

def test_golden_c1_generation(prompt):
    """Regression pin: tokens and exit layers written by tests/golden/make_c1_golden.py (oracle only)."""
    with open(GOLDEN) as f:
        gold = json.load(f)
    m = build_model(C1.shape, C1.weight_seed)
    for tau_s, rec in gold["runs"].items():
        toks, exits = m.generate_g0(prompt, N_NEW, float(tau_s))
        assert toks.tolist() == rec["tokens"] and exits.tolist() == rec["exit_layers"]
