"""Shared test plumbing: loads the seeded workload into the HIP library and into the oracle, and runs
the two in lockstep with the teacher-forcing rule for decisions inside the guard band."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

import paper_2312_04916_amd as ee
from oracle import oracle as O
from workload import ModelShape, model_tensor, model_tensor_list

GUARD = 1e-2  # oracle confidence within this of the threshold, or top-2 logit gap below it: follow the GPU


def ee_config_of(shape: ModelShape, max_positions: int) -> ee.ee_config:
    return ee.make_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff, shape.vocab,
                          shape.exit_layers, shape.dtype, max_positions, shape.rms_eps, shape.rope_base, shape.exit_flags)


def load_gpu_model(shape: ModelShape, seed: int = 0, gain_jitter: float = 0.0, max_positions: int = 256,
                   max_rows: int = 64, max_seqs: int = 1) -> ee.Model:
    """Generates every tensor on the device with the workload generator and hands it to the library."""
    m = ee.Model(ee_config_of(shape, max_positions), max_rows, max_seqs)
    for kind, idx in model_tensor_list(shape):
        t = model_tensor(shape, kind, idx, seed, "cuda:0", gain_jitter).contiguous()
        m.set_tensor(int(kind), idx, t)
        torch.cuda.synchronize()
        del t
    return m


def rel_err(a: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(a.astype(np.float64) - ref.astype(np.float64))) / max(np.max(np.abs(ref)), 1e-30))


@dataclass
class LockstepReport:
    tokens: List[int] = field(default_factory=list)
    exit_layers: List[int] = field(default_factory=list)
    teacher_forced: int = 0
    forced_full: int = 0
    max_hidden_err: float = 0.0
    max_logit_err: float = 0.0
    max_conf_err: float = 0.0
    mismatches: List[str] = field(default_factory=list)


def _judge(rep: LockstepReport, step: int, diag: dict, tau: float, gpu_exits_here: bool, gpu_tok: int, is_final: bool,
           evaluated: bool) -> bool:
    """Compares one head evaluation of the oracle with what the GPU did there.  Returns True when the
    step ends at this head (following the GPU inside the guard band)."""
    if not is_final:
        if not evaluated:
            if gpu_exits_here:
                rep.mismatches.append(f"step {step}: GPU left at layer {diag['layer']} where exits are off")
            return False
        fires = diag["conf"] >= tau
        if fires != gpu_exits_here:
            if abs(diag["conf"] - tau) <= GUARD:
                rep.teacher_forced += 1
            else:
                rep.mismatches.append(f"step {step}: exit decision at layer {diag['layer']} differs "
                                      f"(oracle conf {diag['conf']:.6f}, tau {tau}, gpu exits {gpu_exits_here})")
        if not gpu_exits_here:
            return False
    if gpu_tok != diag["argmax"]:
        gap = diag["top1"] - diag["top2"]
        if gap < GUARD and gpu_tok == diag["arg2"]:
            rep.teacher_forced += 1
        else:
            rep.mismatches.append(f"step {step}: token at layer {diag['layer']} differs (oracle {diag['argmax']}, "
                                  f"gpu {gpu_tok}, top-2 gap {gap:.6f})")
    return True


def lockstep(gm: ee.Model, cache: ee.KvCache, om: O.Model, prompt, n_new: int, tau: float, max_pending: int,
             seq: int = 0, check_hidden: bool = True, logits: Optional[torch.Tensor] = None,
             max_positions: Optional[int] = None) -> LockstepReport:
    """Generates n_new tokens on the GPU and drives the oracle through the same decisions."""
    sh = om.cfg
    L, n_exits = sh.n_layers, sh.n_exits
    rep = LockstepReport()
    st = O.State(om, max_positions or (len(prompt) + n_new + 1), max_pending)

    def check_state(step, diag):
        if check_hidden:
            rep.max_hidden_err = max(rep.max_hidden_err, rel_err(cache.read_hidden(seq), st.last_hidden()))
        if logits is not None:
            rep.max_logit_err = max(rep.max_logit_err, rel_err(logits[0].cpu().numpy(), st.last_logits()))

    # prefill: every head is evaluated on the last prompt position; the rule picks the first token
    diags = st.prefill(prompt)
    tok, ex, conf = ee.prefill(gm, cache, seq, prompt, tau)
    for i, dg in enumerate(diags):
        fin = i == n_exits
        if _judge(rep, 0, dg, tau, ex == dg["layer"], tok, fin, tau < 1.0):
            rep.max_conf_err = max(rep.max_conf_err, abs(float(conf[i]) - dg["conf"]))
            break
    rep.tokens.append(int(tok))
    rep.exit_layers.append(int(ex))
    if check_hidden:  # after prefill both hold the last prompt position at full depth
        rep.max_hidden_err = max(rep.max_hidden_err, rel_err(cache.read_hidden(seq), st.last_hidden()))

    seqs = ee.Sequences(L)
    seqs.start(seq, tok)
    for step in range(1, n_new):
        ro, tk, pm = seqs.rows([seq])
        cur = seqs.current[seq]
        nt, exl, cf = ee.decode_step(gm, cache, [seq], ro, tk, pm, tau)
        g_tok, g_ex = int(nt[0]), int(exl[0])
        forced = st.step_begin(cur)
        rep.forced_full += int(forced)
        evaluated = (not forced) and tau < 1.0
        while True:
            depth, dg = st.step_advance(evaluated)
            fin = depth == L
            if dg is None:
                if g_ex == depth:
                    rep.mismatches.append(f"step {step}: GPU left at layer {depth} where exits are off")
                continue
            if _judge(rep, step, dg, tau, g_ex == depth, g_tok, fin, evaluated):
                rep.max_conf_err = max(rep.max_conf_err, abs(float(cf[0]) - dg["conf"]))
                check_state(step, dg)
                break
            if fin:
                break
        st.step_commit(g_tok)
        seqs.update([seq], nt, exl)
        rep.tokens.append(g_tok)
        rep.exit_layers.append(g_ex)
        if cache.pending(seq) != st.n_pending():
            rep.mismatches.append(f"step {step}: pending {cache.pending(seq)} vs oracle {st.n_pending()}")
    rep.state = st
    rep.seqs = seqs
    return rep


def build_pair(shape: ModelShape, seed: int = 0, gain_jitter: float = 0.0, max_positions: int = 256,
               max_rows: int = 64, max_seqs: int = 1):
    """(oracle model, GPU model) over the same seeded tensors: each tensor is generated once on the device
    (the generator is bit-identical on CPU and GPU), handed to the library, and copied to the host for the
    oracle."""
    from oracle.from_workload import config_of, to_numpy

    om = O.Model(config_of(shape))
    gm = ee.Model(ee_config_of(shape, max_positions), max_rows, max_seqs)
    for kind, idx in model_tensor_list(shape):
        t = model_tensor(shape, kind, idx, seed, "cuda:0", gain_jitter).contiguous()
        gm.set_tensor(int(kind), idx, t)
        om.set_tensor(int(kind), idx, to_numpy(t))
        torch.cuda.synchronize()
        del t
    return om, gm
