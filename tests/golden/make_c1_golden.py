"""Writes tests/golden/c1_generation.json: tokens and exit layers of the tiny fp32 workload, from the
oracle's plain-definition generator only (nothing here touches the HIP library).

The paper prints no worked example that can be reproduced without its trained weights (its Tables 3
and 4 need the trained 7B model and tokenizer), so these stored values are a regression pin of the
oracle, not a citation.   Usage: python tests/golden/make_c1_golden.py
"""
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))

from oracle.from_workload import build_model  # noqa: E402
from workload import CONFIGS, prompt_tokens  # noqa: E402


def main():
    w = CONFIGS["C1"]
    m = build_model(w.shape, w.weight_seed)
    prompt = prompt_tokens(w.shape.vocab, w.prompt_len[0], w.prompt_seed).numpy()
    runs = {}
    for tau in w.thresholds:
        toks, exits = m.generate_g0(prompt, w.new_tokens, tau)
        runs[repr(float(tau))] = {"tokens": toks.tolist(), "exit_layers": exits.tolist()}
    out = {"workload": "C1", "weight_seed": w.weight_seed, "prompt_seed": w.prompt_seed,
           "prompt": prompt.tolist(), "runs": runs}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_generation.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
