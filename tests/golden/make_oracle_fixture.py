"""Writes tests/golden/oracle_config1.json: what the CPU oracle returns for the smallest configuration (d = 256,
N = 1024, k' = 208, k = 52, seeded inputs), so that an unintended change of the oracle's arithmetic shows up as a
diff of this file.  Calls only the oracle and the seeded input generators; run from the repository root:

    python tests/golden/make_oracle_fixture.py
"""
import hashlib
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
from oracle import hire_oracle as O                       # noqa: E402
from paper_2402_09360_amd import inputs as I              # noqa: E402


def fixture():
    O.build()
    d, N, k, kp = 256, 1024, 52, 208
    L = I.ffn_layer(11, d, N)
    x = I.tokens(12, 2, d)
    q, s = O.quantize_rows_int4(L["w1u"])
    out = O.ffn_step(L["w1u"], L["w2u"], ("int4", q, s), x, k, kp, want_acc=True)
    W = I.classifier(13, 3000, d)
    qc, sc = O.quantize_rows_int4(W)
    sm = O.softmax_step(W, ("int4", qc, sc), x, 8, 64)
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    return {
        "ffn": {"d": d, "N": N, "k": k, "kprime": kp, "seeds": {"layer": 11, "tokens": 12},
                "scale_sha256": sha(s), "codes_sha256": sha(q), "acc_sha256": sha(out["acc"]),
                "cand": out["cand"].tolist(), "topk_idx": out["topk_idx"].tolist(),
                "y_first8": [float(v) for v in out["y"][0, :8]], "y_sha256_of_float32": sha(out["y"].astype(np.float32))},
        "softmax": {"d": d, "classes": 3000, "k": 8, "kprime": 64, "seeds": {"classifier": 13, "tokens": 12},
                    "top_idx": sm["top_idx"].tolist(), "top_prob": [[float(v) for v in row] for row in sm["top_prob"]]},
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_config1.json")
    fx = fixture()
    with open(path, "w") as f:   # one key per line: short, and a change shows up as a one-line diff
        f.write("{\n")
        for i, part in enumerate(sorted(fx)):
            f.write(f' "{part}": {{\n')
            keys = sorted(fx[part])
            for j, key in enumerate(keys):
                f.write(f'  "{key}": {json.dumps(fx[part][key], sort_keys=True)}{"," if j + 1 < len(keys) else ""}\n')
            f.write(" }" + ("," if i + 1 < len(fx) else "") + "\n")
        f.write("}\n")
    print("wrote", path)
