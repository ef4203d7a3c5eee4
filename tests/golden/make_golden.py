"""Writes the stored expected values under tests/golden/ by calling only the
float64 oracle.  Run from the repository root:  python tests/golden/make_golden.py

accept_v4_example.json -- a four-token position with a drafter that prefers a
different token than the target (T = 1, eta = 2, tail 0.1).  The paper prints no
worked numbers; this fixture records the oracle's output for Eq. new_target, the
tail rule and Alg. 1's accept/residual on that input so that later edits of the
oracle are noticed.  The test that reads it re-derives every number with library
softmax arithmetic as well.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def main():
    z, zq, eta, T, alpha = [2.0, 1.0, 0.0, -1.0], [0.0, 2.0, 1.0, -1.0], 2.0, 1.0, 0.1
    p, q, ph = oracle.distributions(z, zq, eta=eta, temperature=T, tail_alpha=alpha)
    acc = np.minimum(q, ph)
    beta = float(acc.sum())
    w = np.maximum(np.maximum(p - ph, p - q), 0.0)
    law = acc + (1 - beta) * w / w.sum()
    cases = []
    for draft, r, u in [(1, 0.5, 0.3), (1, 0.95, 0.3), (0, 0.5, 0.99), (2, 0.7, 0.5), (2, 0.5, 0.5)]:
        res = oracle.accept(np.array([[z, z]], np.float32), np.array([[zq]], np.float32),
                            np.array([[draft]], np.int32), np.array([[r, u]], np.float32), eta=eta)
        cases.append({"draft": draft, "r": r, "u": u, "n_accepted": int(res.n_accepted[0]),
                      "token": int(res.out_tokens[0, 0])})
    out = {"source": "oracle/rapid_oracle.c via tests/golden/make_golden.py",
           "z": z, "zq": zq, "eta": eta, "T": T, "tail_alpha": alpha,
           "p": p.tolist(), "q": q.tolist(), "p_hat": ph.tolist(), "beta": beta,
           "residual_weights": w.tolist(), "law": law.tolist(), "cases": cases}
    with open(os.path.join(HERE, "accept_v4_example.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
