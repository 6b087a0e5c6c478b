"""Writes tests/golden/cfg1_oracle.json: the oracle's own results on the tiny workload (argmax,
accepted path, a few logits).  Calls only oracle/ and the seeded input generators; a regression
guard for the oracle, not a paper value (the paper prints no worked example)."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workload as wl  # noqa: E402


def compute():
    spec = wl.WORKLOADS["cfg1_tiny"]
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, spec["seed"], "f32")
    audio, text = wl.make_prefix_inputs(cfg, spec["seed"], spec["n_audio"], spec["n_text"])
    parents, tokens = wl.make_tree("cfg1_tiny")
    om = oracle.OracleModel(cfg, w)
    kc, vc = om.empty_cache(96)
    L, _ = om.prefill(kc, vc, 0, audio.astype(np.float64), text)
    r = om.tree_forward(kc, vc, L, tokens, parents)
    path, alen, nxt = oracle.accept(tokens, parents, r["amax"])
    return dict(kv_len=int(L), tokens=tokens.tolist(), parents=parents.tolist(),
                amax=r["amax"].tolist(), path=path.tolist(), accept_len=alen, next_token=nxt,
                logits_node0_first8=[float("%.12e" % v) for v in r["logits"][0, :8]],
                logits_node7_first8=[float("%.12e" % v) for v in r["logits"][7, :8]])


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.json")
    json.dump(compute(), open(out, "w"), indent=1)
    print("wrote", out)
