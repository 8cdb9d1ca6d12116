"""GPU parity of the prompt phase through the GEMM path (bf16 models, prompts of 32 tokens or more) and of
the heads scored on every position, through the C ABI, against the CPU oracle's cache-free forward of the
whole sequence: cached K and V of every layer and the last hidden state within 2e-3 relative, first token
and exit layer by the exit rule, per-position arg max exact outside the guard band, confidences within 2e-3."""
import os

import numpy as np
import pytest
import scipy.special

import paper_2312_04916_amd as ee
from oracle.from_workload import build_model
from workload import ModelShape, prompt_tokens

from common import GUARD, TOL, TOL_CONF, TOL_CONF_ONE_TERM, TOL_NLL_ONE_TERM, flip_guard, kv_check, load_gpu_model, rel_err

pytestmark = pytest.mark.gpu

SHAPES = {
    "hd32": ModelShape(4, 128, 4, 32, 352, 1024, (1, 2), "bf16", 0.02, 0.3),
    "hd64": ModelShape(3, 256, 4, 64, 512, 2048, (1, 2), "bf16", 0.02, 0.3 / 2 ** 0.5),
    "hd128": ModelShape(3, 256, 2, 128, 544, 2080, (2,), "bf16", 0.02, 0.3 / 2 ** 0.5),
}


def oracle_scores(om, shape, hid, n):
    """Per head and position: (arg max, confidence, second candidate, top-2 gap) from the oracle's hidden states."""
    heads = list(shape.exit_layers) + [shape.n_layers]
    out = []
    for hi, layer in enumerate(heads):
        rows = []
        for p in range(n):
            _, dg = om.head_row(hi, hid[layer][p])
            rows.append(dg)
        out.append(rows)
    return out


def check_prefill(shape, n_prompt, seed, rows_env=None, scored=True, tau=0.35, head_terms=2):
    """head_terms: ee_config::scored_head_terms.  2 = the scored heads take both bf16 terms of their input, like every
    other GEMM, and are held to the tolerances of the decode heads; 1 (the library's default) = the leading term only."""
    om = build_model(shape, seed, gain_jitter=0.1)
    gm = load_gpu_model(shape, seed, gain_jitter=0.1, max_positions=512, max_rows=64, max_seqs=1, prefill_rows=rows_env or 0,
                        scored_head_terms=head_terms)
    tol_pos = TOL_CONF["bf16"] if head_terms == 2 else TOL_CONF_ONE_TERM
    p = prompt_tokens(shape.vocab, n_prompt, 40 + seed).numpy()
    cache = ee.KvCache(gm, 1, 512, 64, 8)
    hid, ko, vo = om.forward_sequence(p)
    if scored:
        tok, ex, conf, ptok, pconf = ee.prefill_scored(gm, cache, 0, p, tau)
    else:
        tok, ex, conf = ee.prefill(gm, cache, 0, p, tau)
    L = shape.n_layers
    for l in range(L):
        assert cache.filled(0, l) == n_prompt
        k, v = cache.read(0, l, 0, n_prompt)
        kv_check(k, ko[l], "bf16", "K", l), kv_check(v, vo[l], "bf16", "V", l)
    herr = rel_err(cache.read_hidden(0), hid[L][n_prompt - 1])
    assert herr <= TOL["bf16"], herr
    sc = oracle_scores(om, shape, hid, n_prompt)
    # the first generated token: shallowest exit whose confidence passes, else the final head
    chosen = len(sc) - 1
    for hi in range(len(sc) - 1):
        dg = sc[hi][n_prompt - 1]
        fires = dg["conf"] >= tau
        if abs(dg["conf"] - tau) <= GUARD:
            fires = ex == shape.exit_layers[hi]  # inside the guard band: follow the GPU
        if fires:
            chosen = hi
            break
    heads = list(shape.exit_layers) + [L]
    assert ex == heads[chosen], (ex, heads[chosen])
    dg = sc[chosen][n_prompt - 1]
    assert tok == dg["argmax"] or (dg["top1"] - dg["top2"] < GUARD and tok == dg["arg2"])
    for hi in range(len(sc)):
        assert abs(float(conf[hi]) - sc[hi][n_prompt - 1]["conf"]) <= TOL_CONF["bf16"]
    forced = 0
    if scored:
        for hi in range(len(sc)):
            for pos in range(n_prompt):
                dg = sc[hi][pos]
                if int(ptok[hi, pos]) != dg["argmax"]:
                    assert dg["top1"] - dg["top2"] < flip_guard(dg, head_terms) and int(ptok[hi, pos]) == dg["arg2"], (hi, pos, dg, int(ptok[hi, pos]))
                    forced += 1
                assert abs(float(pconf[hi, pos]) - dg["conf"]) <= tol_pos, (hi, pos, float(pconf[hi, pos]), dg["conf"])
        # the last position repeats what the rule saw (the rule's heads always take both terms)
        for hi in range(len(sc)):
            assert abs(float(pconf[hi, n_prompt - 1]) - float(conf[hi])) <= (1e-4 if head_terms == 2 else TOL_CONF_ONE_TERM)
    print(f"prefill {shape.d_model}/{shape.head_dim} n={n_prompt} rows_env={rows_env} head terms {head_terms}: hidden err {herr:.2e}, "
          f"guard-band positions {forced}", flush=True)
    cache.close()
    gm.close()


@pytest.mark.parametrize("name,n", [("hd32", 150), ("hd64", 333), ("hd128", 200), ("hd32", 32), ("hd128", 128)])
def test_prefill_gemm_path_and_scored_heads(name, n):
    print(f"case: prefill scored {name} n={n}", flush=True)
    check_prefill(SHAPES[name], n, 1)


@pytest.mark.parametrize("name,n", [("hd32", 150), ("hd64", 333), ("hd128", 128)])
def test_scored_heads_on_the_leading_term(name, n):
    """The library's default for the scored heads: the leading bf16 term of their input only."""
    print(f"case: prefill scored, one-term heads {name} n={n}", flush=True)
    check_prefill(SHAPES[name], n, 1, head_terms=1)


def test_prefill_in_several_passes():
    """Prompt longer than one pass (128 rows): later passes attend to the cache the earlier ones wrote."""
    print("case: prefill passes", flush=True)
    check_prefill(SHAPES["hd64"], 300, 2, rows_env=128)


def test_prefill_plain_entry_takes_the_same_path():
    print("case: prefill plain", flush=True)
    check_prefill(SHAPES["hd32"], 97, 3, scored=False)


def test_scored_short_prompt_and_path_switched_off():
    """A scored prompt shorter than 32 tokens still goes through the GEMM path; with the path switched off the
    scored entry point reports a configuration error and the plain one still works (decode kernels)."""
    print("case: prefill short / off", flush=True)
    check_prefill(SHAPES["hd32"], 7, 4)
    shape = SHAPES["hd32"]
    gm = load_gpu_model(shape, 4, gain_jitter=0.1, max_positions=256, max_rows=64, max_seqs=1, prefill_rows=-1)
    cache = ee.KvCache(gm, 1, 256, 32, 8)
    p = prompt_tokens(shape.vocab, 50, 44).numpy()
    with pytest.raises(ee.EeError) as e:
        ee.prefill_scored(gm, cache, 0, p, 0.5)
    assert e.value.code == -1
    tok, ex, conf = ee.prefill(gm, cache, 0, p, 0.5)
    assert cache.filled(0, shape.n_layers - 1) == 50
    cache.close()
    gm.close()


@pytest.mark.parametrize("name,n,rows_env,head_terms", [("hd64", 210, None, 2), ("hd32", 300, 128, 2), ("hd64", 210, None, 1)])
def test_scored_negative_log_likelihood_of_the_prompt(name, n, rows_env, head_terms):
    """pos_nll[i][t] = -log p_i(tokens[t+1] | tokens[..t]) of every head: the per-token cross-entropy terms of the
    early-exit training objective (Section 3, Eq. (1)), against log-sum-exp (scipy, fp64) of the oracle's logits.
    With rows_env the prompt spans several passes: the target of a pass's last row is the next pass's first token."""
    print(f"case: scored nll {name} n={n} rows_env={rows_env} head terms {head_terms}", flush=True)
    shape = SHAPES[name]
    om = build_model(shape, 5, gain_jitter=0.1)
    gm = load_gpu_model(shape, 5, gain_jitter=0.1, max_positions=512, max_rows=64, max_seqs=1, prefill_rows=rows_env or 0,
                        scored_head_terms=head_terms)
    tol_nll = TOL["bf16"] if head_terms == 2 else TOL_NLL_ONE_TERM
    p = prompt_tokens(shape.vocab, n, 45).numpy()
    cache = ee.KvCache(gm, 1, 512, 64, 8)
    hid, _, _ = om.forward_sequence(p)
    out = ee.prefill_scored(gm, cache, 0, p, 0.5, nll=True)
    pnll, pconf = out[5], out[4]
    heads = list(shape.exit_layers) + [shape.n_layers]
    worst = 0.0
    for hi, layer in enumerate(heads):
        for pos in range(n - 1):
            z, dg = om.head_row(hi, hid[layer][pos])
            ref = float(scipy.special.logsumexp(z.astype(np.float64)) - float(z[p[pos + 1]]))
            got = float(pnll[hi, pos])
            worst = max(worst, abs(got - ref))
            assert abs(got - ref) <= tol_nll * max(1.0, abs(ref)), (hi, pos, got, ref)
            # consistency with the confidence of the same head: -log(conf) = log-sum-exp - max logit
            lse = float(scipy.special.logsumexp(z.astype(np.float64)))
            assert abs(-np.log(float(pconf[hi, pos])) - (lse - dg["top1"])) <= (TOL_CONF["bf16"] if head_terms == 2 else tol_nll * max(1.0, abs(lse)))
        assert pnll[hi, n - 1] == 0.0  # no token follows the last position
    assert float(np.mean(pnll[:, :-1])) > 1.0  # random weights: the mean loss is of the order of log(vocab)
    print(f"  worst |nll - oracle| = {worst:.2e}, mean nll {np.mean(pnll[:, :-1]):.3f}", flush=True)
    cache.close()
    gm.close()
