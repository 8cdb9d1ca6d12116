"""Pins of the oracle's exit structures (Section 2, "Model architectures": an output embedding matrix, an
optional normalisation in front of it, optionally an MLP before that, embeddings tied or untied) against numpy
fp64 formulas, special cases that reduce to the already pinned default exit, and the statement that the output
does not depend on the inference method (Appendix B.1).  CPU only.
"""
import dataclasses

import numpy as np
import pytest
import scipy.special

from oracle import oracle as O
from oracle.from_workload import build_model, to_numpy
from workload import CONFIGS, ModelShape, TensorKind, model_tensor, model_tensor_list, prompt_tokens

BASE = ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "f32", 0.02, 0.3)
RNG = np.random.default_rng(99)


def variant(**kw) -> ModelShape:
    return dataclasses.replace(BASE, **kw)


def x_row(scale=1.0):
    return np.ascontiguousarray(RNG.standard_normal(BASE.d_model) * scale, dtype=np.float32)


def rms(x, g, eps):
    x = x.astype(np.float64)
    return x * g.astype(np.float64) / np.sqrt(np.mean(x * x) + eps)


def test_exit_flags_and_tensor_lists():
    assert BASE.exit_flags == 0
    assert variant(exit_norm=False).exit_flags == 1
    assert variant(tie_embeddings=True).exit_flags == 2
    assert variant(exit_mlp=True).exit_flags == 4
    kinds = [k for k, _ in model_tensor_list(variant(exit_norm=False, tie_embeddings=True))]
    assert TensorKind.EXIT_NORM not in kinds and TensorKind.EXIT_HEAD not in kinds and TensorKind.FINAL_HEAD not in kinds
    assert TensorKind.FINAL_NORM in kinds
    kinds = [k for k, _ in model_tensor_list(variant(exit_mlp=True))]
    assert kinds.count(TensorKind.EXIT_WG) == 2 and kinds.count(TensorKind.EXIT_MLP_NORM) == 2
    # the default model's tensors are what they were before the exit structures existed
    assert [k for k, _ in model_tensor_list(BASE)].count(TensorKind.EXIT_HEAD) == 2


def test_exit_without_norm_is_a_plain_matvec_and_scales_with_its_input():
    sh = variant(exit_norm=False)
    m = build_model(sh, 3, gain_jitter=0.1)
    x = x_row(2.0)
    for e in range(2):
        z, dg = m.head_row(e, x)
        W = m.tensor(TensorKind.EXIT_HEAD, e).astype(np.float64)
        ref = W @ x.astype(np.float64)
        assert np.max(np.abs(z - ref)) <= 1e-6 * np.max(np.abs(ref))
        assert dg["argmax"] == int(np.argmax(ref))
        # no normalisation: doubling the input doubles the logits (a normalised exit would not move)
        z2, _ = m.head_row(e, (2 * x).astype(np.float32))
        assert np.max(np.abs(z2 - 2 * z)) <= 1e-5 * np.max(np.abs(z))
    # the final head keeps its norm: scale-invariant
    zf, _ = m.head_row(2, x)
    zf2, _ = m.head_row(2, (2 * x).astype(np.float32))
    assert np.max(np.abs(zf2 - zf)) <= 1e-4 * np.max(np.abs(zf))
    g = m.tensor(TensorKind.FINAL_NORM, 0)
    ref = m.tensor(TensorKind.FINAL_HEAD, 0).astype(np.float64) @ rms(x, g, sh.rms_eps)
    assert np.max(np.abs(zf - ref)) <= 1e-5 * np.max(np.abs(ref))


def test_tied_heads_read_the_embedding_matrix():
    sh = variant(tie_embeddings=True)
    m = build_model(sh, 4, gain_jitter=0.1)
    E = m.tensor(TensorKind.EMBED, 0).astype(np.float64)
    x = x_row()
    for h in range(3):
        z, dg = m.head_row(h, x)
        g = m.tensor(TensorKind.FINAL_NORM, 0) if h == 2 else m.tensor(TensorKind.EXIT_NORM, h)
        ref = E @ rms(x, g, sh.rms_eps)
        assert np.max(np.abs(z - ref)) <= 1e-5 * np.max(np.abs(ref))
        p = scipy.special.softmax(ref)
        assert abs(dg["conf"] - p.max()) <= 1e-5
    # the same model written untied, with copies of the embedding as heads, generates the same tokens
    untied = O.Model(O.make_config(sh.n_layers, sh.d_model, sh.n_heads, sh.head_dim, sh.d_ff, sh.vocab, sh.exit_layers,
                                   sh.dtype, sh.rms_eps, sh.rope_base, 0))
    for kind, idx in model_tensor_list(sh):
        untied.set_tensor(kind, idx, m.tensor(kind, idx))
    for e in range(2):
        untied.set_tensor(TensorKind.EXIT_HEAD, e, m.tensor(TensorKind.EMBED, 0).copy())
    untied.set_tensor(TensorKind.FINAL_HEAD, 0, m.tensor(TensorKind.EMBED, 0).copy())
    p = prompt_tokens(sh.vocab, 12, 5).numpy()
    for tau in (0.0, 0.1, 1.0):
        t0, e0 = m.generate_g0(p, 12, tau)
        t1, e1 = untied.generate_g0(p, 12, tau)
        assert np.array_equal(t0, t1) and np.array_equal(e0, e1)


def test_exit_mlp_matches_fp64_formula_and_leaves_the_backbone_alone():
    sh = variant(exit_mlp=True)
    m = build_model(sh, 5, gain_jitter=0.1)
    x = x_row(1.5)
    for e in range(2):
        z, _ = m.head_row(e, x)
        gm = m.tensor(TensorKind.EXIT_MLP_NORM, e)
        Wg, Wu, Wd = (m.tensor(k, e).astype(np.float64) for k in (TensorKind.EXIT_WG, TensorKind.EXIT_WU, TensorKind.EXIT_WD))
        h = rms(x, gm, sh.rms_eps)
        gate, up = Wg @ h, Wu @ h
        x1 = x.astype(np.float64) + Wd @ (gate / (1.0 + np.exp(-gate)) * up)
        ref = m.tensor(TensorKind.EXIT_HEAD, e).astype(np.float64) @ rms(x1.astype(np.float32), m.tensor(TensorKind.EXIT_NORM, e), sh.rms_eps)
        assert np.max(np.abs(z - ref)) <= 2e-5 * np.max(np.abs(ref))
        # a mistake that skipped the residual connection or the block would be far off
        plain = m.tensor(TensorKind.EXIT_HEAD, e).astype(np.float64) @ rms(x, m.tensor(TensorKind.EXIT_NORM, e), sh.rms_eps)
        assert np.max(np.abs(z - plain)) > 1e-3 * np.max(np.abs(ref))
    # the final head has no MLP of its own
    zf, _ = m.head_row(2, x)
    ref = m.tensor(TensorKind.FINAL_HEAD, 0).astype(np.float64) @ rms(x, m.tensor(TensorKind.FINAL_NORM, 0), sh.rms_eps)
    assert np.max(np.abs(zf - ref)) <= 1e-5 * np.max(np.abs(ref))
    # exits off (threshold 1): the tokens are those of the model without the exit MLPs (same backbone tensors)
    base = build_model(BASE, 5, gain_jitter=0.1)
    p = prompt_tokens(sh.vocab, 10, 6).numpy()
    assert np.array_equal(m.generate_g0(p, 10, 1.0)[0], base.generate_g0(p, 10, 1.0)[0])
    hid_m, k_m, _ = m.forward_sequence(p)
    hid_b, k_b, _ = base.forward_sequence(p)
    assert np.array_equal(hid_m, hid_b) and np.array_equal(k_m, k_b)


def test_exit_mlp_with_zero_down_projection_is_the_default_exit():
    sh = variant(exit_mlp=True)
    m = build_model(sh, 6, gain_jitter=0.1)
    base = build_model(BASE, 6, gain_jitter=0.1)
    for e in range(2):
        m.set_tensor(TensorKind.EXIT_WD, e, np.zeros((sh.d_model, sh.d_ff), np.float32))
    x = x_row()
    for e in range(2):
        assert np.array_equal(m.head_row(e, x)[0], base.head_row(e, x)[0])


@pytest.mark.parametrize("kw", [dict(exit_norm=False), dict(tie_embeddings=True), dict(exit_mlp=True),
                                dict(exit_norm=False, tie_embeddings=True, exit_mlp=True)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_kv_recomputation_equals_the_plain_definition_for_every_exit_structure(kw, dtype):
    sh = variant(dtype=dtype, **kw)
    if sh.tie_embeddings:
        sh = dataclasses.replace(sh, head_sigma=0.5)
    m = build_model(sh, 7, gain_jitter=0.1)
    p = prompt_tokens(sh.vocab, 14, 8).numpy()
    mixes = set()
    for tau in (0.0, 0.05, 0.2, 0.5, 1.0):
        t0, e0 = m.generate_g0(p, 20, tau)
        st = O.State(m, 64, 0)
        diags = st.prefill(p)
        tok, ex = diags[-1]["argmax"], diags[-1]["layer"]
        if tau < 1.0:
            for dg in diags[:-1]:
                if dg["conf"] >= tau:
                    tok, ex = dg["argmax"], dg["layer"]
                    break
        toks, exits = [tok], [ex]
        for _ in range(19):
            tok, ex, _ = st.decode_step(tok, tau)
            toks.append(tok)
            exits.append(ex)
        assert np.array_equal(t0, toks) and np.array_equal(e0, exits)
        mixes.update(exits)
    assert len(mixes) >= 2, "the thresholds must exercise exits and the final head"


# ---------------------------------------------------------------- a complete Transformer layer in the exit

def _np_block(x, K, V, w, H, hd, eps, base):
    """One pre-norm block on one row in numpy fp64 (K, V: rows of the earlier positions, this row appended)."""
    pos = len(K)
    d = len(x)
    h = rms(x.astype(np.float32), w["g1"], eps)
    q, k, v = w["wq"] @ h, w["wk"] @ h, w["wv"] @ h

    def rot(vec):
        out = vec.copy()
        half = hd // 2
        for hh in range(H):
            for i in range(half):
                ang = pos * base ** (-2.0 * i / hd)
                a, b = vec[hh * hd + i], vec[hh * hd + i + half]
                out[hh * hd + i] = a * np.cos(ang) - b * np.sin(ang)
                out[hh * hd + i + half] = b * np.cos(ang) + a * np.sin(ang)
        return out

    q, k = rot(q), rot(k)
    K.append(k)
    V.append(v)
    Ka, Va = np.array(K), np.array(V)
    a = np.zeros(d)
    for hh in range(H):
        sl = slice(hh * hd, (hh + 1) * hd)
        p = scipy.special.softmax(Ka[:, sl] @ q[sl] / np.sqrt(hd))
        a[sl] = p @ Va[:, sl]
    x1 = x + w["wo"] @ a
    h2 = rms(x1.astype(np.float32), w["g2"], eps)
    gate, up = w["wg"] @ h2, w["wu"] @ h2
    return x1 + w["wd"] @ (gate / (1.0 + np.exp(-gate)) * up)


def _exit_w(m, e):
    names = dict(g1=TensorKind.EXIT_ATTN_NORM, wq=TensorKind.EXIT_WQ, wk=TensorKind.EXIT_WK, wv=TensorKind.EXIT_WV,
                 wo=TensorKind.EXIT_WO, g2=TensorKind.EXIT_MLP_NORM, wg=TensorKind.EXIT_WG, wu=TensorKind.EXIT_WU,
                 wd=TensorKind.EXIT_WD)
    return {k: m.tensor(v, e).astype(np.float64) for k, v in names.items()}


def test_exit_layer_flags_and_tensor_list():
    sh = variant(exit_layer=True)
    assert sh.exit_flags == 8
    kinds = [k for k, _ in model_tensor_list(sh)]
    for k in (TensorKind.EXIT_ATTN_NORM, TensorKind.EXIT_WQ, TensorKind.EXIT_WK, TensorKind.EXIT_WV, TensorKind.EXIT_WO,
              TensorKind.EXIT_MLP_NORM, TensorKind.EXIT_WG, TensorKind.EXIT_WU, TensorKind.EXIT_WD):
        assert kinds.count(k) == 2
    # an exit cannot have both an MLP of its own and a layer of its own (the layer already ends in an MLP)
    with pytest.raises(ValueError):
        O.Model(O.make_config(4, 128, 4, 32, 352, 1024, (1, 2), "f32", exit_flags=4 | 8))


def test_exit_layer_matches_a_numpy_fp64_block_over_the_sequence():
    """The exit's layer is an ordinary causal Transformer block over the hidden states at the exit's depth: against a
    block written out in numpy fp64 (its own attention over its own keys and values), then the exit's norm and head."""
    sh = variant(exit_layer=True)
    m = build_model(sh, 11, gain_jitter=0.1)
    n = 7
    hid = np.ascontiguousarray(RNG.standard_normal((n, sh.d_model)), dtype=np.float32)
    for e in range(2):
        xo, ko, vo = m.exit_layer_sequence(e, hid)
        w = _exit_w(m, e)
        K, V = [], []
        for t in range(n):
            ref = _np_block(hid[t].astype(np.float64), K, V, w, sh.n_heads, sh.head_dim, sh.rms_eps, sh.rope_base)
            assert np.max(np.abs(xo[t] - ref)) <= 2e-5 * np.max(np.abs(ref)), (e, t)
        assert np.max(np.abs(ko - np.array(K))) <= 1e-5 * np.max(np.abs(K))
        assert np.max(np.abs(vo - np.array(V))) <= 1e-5 * np.max(np.abs(V))
        # the last position really attends to the earlier ones: changing position 0 changes it
        hid2 = hid.copy()
        hid2[0] += 1.0
        xo2, _, _ = m.exit_layer_sequence(e, hid2)
        assert np.max(np.abs(xo2[-1] - xo[-1])) > 1e-4
        # ... and never to later ones (causal)
        hid3 = hid.copy()
        hid3[-1] += 1.0
        xo3, _, _ = m.exit_layer_sequence(e, hid3)
        assert np.array_equal(xo3[:-1], xo[:-1])
        # what follows the layer is the exit's norm and output embedding
        z, _ = m.head_row(e, xo[-1])
        refz = m.tensor(TensorKind.EXIT_HEAD, e).astype(np.float64) @ rms(xo[-1], m.tensor(TensorKind.EXIT_NORM, e), sh.rms_eps)
        assert np.max(np.abs(z - refz)) <= 1e-5 * np.max(np.abs(refz))


def test_exit_layer_with_zero_output_projections_is_the_default_exit():
    """W_o = 0 and W_d = 0 in the exit's layer: the layer adds nothing to x, so tokens, exit layers and the backbone's
    cache are those of the model with the minimalistic exit, for both generators."""
    sh = variant(exit_layer=True)
    m = build_model(sh, 12, gain_jitter=0.1)
    base = build_model(BASE, 12, gain_jitter=0.1)
    for e in range(2):
        m.set_tensor(TensorKind.EXIT_WO, e, np.zeros((sh.d_model, sh.d_model), np.float32))
        m.set_tensor(TensorKind.EXIT_WD, e, np.zeros((sh.d_model, sh.d_ff), np.float32))
    p = prompt_tokens(sh.vocab, 12, 9).numpy()
    for tau in (0.0, 0.15, 0.4, 1.0):
        assert all(np.array_equal(a, b) for a, b in zip(m.generate_g0(p, 14, tau), base.generate_g0(p, 14, tau)))
        outs = []
        for mod in (m, base):
            st = O.State(mod, 64, 3)
            diags = st.prefill(p)
            tok = next((dg["argmax"] for dg in diags[:-1] if tau < 1.0 and dg["conf"] >= tau), diags[-1]["argmax"])
            seq = [tok]
            for _ in range(13):
                tok, ex, _ = st.decode_step(tok, tau)
                seq.append((tok, ex))
            st.flush()
            outs.append((seq, st.kv_read(3, 0, 12 + 13)))
        assert outs[0][0] == outs[1][0]
        assert np.array_equal(outs[0][1][0], outs[1][1][0]) and np.array_equal(outs[0][1][1], outs[1][1][1])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cap", [0, 3])
def test_exit_layer_kv_recomputation_equals_the_plain_definition(dtype, cap):
    """G1 (cache, deferred tokens, the exit layers' own caches filled as positions pass their depth) against G0 (every
    token from a cache-free forward, the exit's layer run over the whole sequence), bit for bit; and after a flush the
    exit layers' caches equal the exit layer applied to the full-depth hidden states of everything generated."""
    sh = variant(dtype=dtype, exit_layer=True)
    m = build_model(sh, 13, gain_jitter=0.1)
    p = prompt_tokens(sh.vocab, 14, 8).numpy()
    mixes = set()
    for tau in (0.0, 0.08, 0.25, 1.0):
        t0, e0 = m.generate_g0(p, 18, tau, max_pending=cap)
        st = O.State(m, 64, cap)
        diags = st.prefill(p)
        tok, ex = diags[-1]["argmax"], diags[-1]["layer"]
        if tau < 1.0:
            for dg in diags[:-1]:
                if dg["conf"] >= tau:
                    tok, ex = dg["argmax"], dg["layer"]
                    break
        toks, exits = [tok], [ex]
        for _ in range(17):
            tok, ex, _ = st.decode_step(tok, tau)
            toks.append(tok)
            exits.append(ex)
        assert np.array_equal(t0, toks) and np.array_equal(e0, exits), (tau, t0, toks, e0, exits)
        mixes.update(exits)
        st.flush()
        seq = np.concatenate([p, np.array(toks[:-1], np.int32)])
        hid, _, _ = m.forward_sequence(seq)
        for e, layer in enumerate(sh.exit_layers):
            _, ke, ve = m.exit_layer_sequence(e, hid[layer])
            kc, vc = st.kv_read(sh.n_layers + e, 0, len(seq))
            assert np.array_equal(kc, ke) and np.array_equal(vc, ve), (tau, e)
    assert len(mixes) >= 2
