"""Writes tiny_config_run.json: the fp32 oracle's greedy run on the tiny
2-layer configuration (weights seed 0, 10-token prompt seed 0, prefill + 16
decode steps).  Calls only oracle/ and the input generators; rerun it only
when the oracle's arithmetic is deliberately changed.

    python tests/golden/make_tiny_golden.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle.cpu_oracle import Oracle                      # noqa: E402
from paper_2604_23467_amd import workloads as wl          # noqa: E402


def main():
    meta = dict(max_seq=64, weight_seed=0, token_seed=0, prompt_len=10, decode_steps=16)
    cfg = wl.tiny_cfg(max_seq=meta["max_seq"])
    w = wl.make_weights_numpy(cfg, seed=meta["weight_seed"])
    prompt = wl.make_tokens(meta["prompt_len"], cfg["vocab"], seed=meta["token_seed"])
    m = Oracle("f32").model(cfg, w)
    t, logits, _ = m.prefill(prompt)
    toks, sums, margins = [t], [float(np.abs(logits).sum())], []
    top2 = np.sort(logits)[-2:]
    margins.append(float(top2[1] - top2[0]))
    for _ in range(meta["decode_steps"]):
        t, logits, _ = m.step(t)
        toks.append(t)
        sums.append(float(np.abs(logits).sum()))
        top2 = np.sort(logits)[-2:]
        margins.append(float(top2[1] - top2[0]))
    meta.update(prompt=prompt.tolist(), tokens=toks, logit_abs_sums=sums, top2_margins=margins,
                _source="written by tests/golden/make_tiny_golden.py from the fp32 CPU oracle")
    json.dump(meta, open(os.path.join(HERE, "tiny_config_run.json"), "w"), indent=1)
    print(toks)


if __name__ == "__main__":
    main()
