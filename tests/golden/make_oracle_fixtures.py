"""Writes tests/golden/oracle_regression.json from the CPU oracle alone (nothing of the GPU path is
imported).  The paper prints no worked numerical example, so these are not the paper's values: they
record what the pinned oracle computes on three small seeded cases, and the test that reads them
fails when a later edit changes the oracle's arithmetic without saying so.

    python tests/golden/make_oracle_fixtures.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import seeded_inputs as si  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_regression.json")


def cases():
    """The three cases, recomputed from seeds.  Used by this script and by the test."""
    out = {}
    # (1) verify pass of the tiny fp32 target over a 12-token prompt (Section 4.1: one causal forward)
    tw = si.decoder_weights(si.TINY_TARGET, 0)
    ot = oracle.Model(si.TINY_TARGET, tw)
    prompt = si.token_ids(0, "golden_prompt", (12,), si.TINY_TARGET.vocab).numpy().tolist()
    logits = np.asarray(ot.forward(ot.new_kv(32), prompt), dtype=np.float64)
    out["forward"] = {
        "prompt": prompt,
        "rows": {str(r): {"first8": [float(x) for x in logits[r, :8]], "sum": float(logits[r].sum()),
                          "argmax": int(np.argmax(logits[r]))} for r in (0, 5, 11)},
    }
    # (2) the modified rejection step on seeded logits (Section 3): batch 6, K 4, vocabulary 50, T 0.7
    p_l, q_l, u, _ = si.accept_workload(7, 6, 4, 50)
    p, q = oracle.softmax(p_l.numpy(), 0.7), oracle.softmax(q_l.numpy(), 0.7)
    ud = si.uniforms(7, "golden_draft", (6, 4)).numpy()
    draft = np.array([[oracle.sample(q[b, i], ud[b, i]) for i in range(4)] for b in range(6)], dtype=np.int32)
    na, nx = oracle.speculative_accept(p, q, draft, u.numpy())
    out["accept"] = {"draft": draft.tolist(), "n_accepted": na.tolist(), "next": nx.tolist(),
                     "p_row0_first4": [float(x) for x in p[0, 0, :4]]}
    # (3) the whole loop (Sections 3 and 4.3): tiny pair, K 3, temperature 1, 24 new tokens
    od = oracle.Model(si.TINY_DRAFT, si.decoder_weights(si.TINY_DRAFT, 100))
    n_new, K = 24, 3
    u_d = si.uniforms(1, "golden_ud", (n_new, K)).numpy()
    u_a = si.uniforms(1, "golden_ua", (n_new, K + 1)).numpy()
    tokens, stats = oracle.speculative_generate(ot, od, prompt, n_new, K, 1.0, u_d, u_a)
    out["loop"] = {"tokens": [int(t) for t in tokens], "accepted": [int(a) for a in stats["accepted"]]}
    return out


if __name__ == "__main__":
    with open(OUT, "w") as f:
        json.dump(cases(), f, indent=1)
        f.write("\n")
    print(OUT)
