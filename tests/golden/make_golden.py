"""Writes tests/golden/opt125m_linear_oracle.txt from the CPU oracle alone.

The paper prints no worked numerical example of the W8A8 operator, so this
fixture is not a paper value: it freezes what the pinned oracle produces for the
OPT-125m-shaped linear (seed 0), so that a later edit of the oracle's arithmetic
cannot pass unnoticed.  Run:  python tests/golden/make_golden.py
Calls only haq_inputs (input generator) and oracle/.
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import haq_inputs as hi  # noqa: E402
import oracle  # noqa: E402


def compute():
    wl = hi.OPT125M_LINEAR
    X, _, _ = hi.hidden_states(wl.seed, wl.T, wl.K, wl.n_outlier, wl.mult)
    W = hi.gaussian_weight(wl.seed, 0, wl.K, wl.N)
    s = oracle.smoothing_vector(oracle.col_absmax_f16(X), oracle.row_absmax_f32(W), 0.5)
    Wq, sw = oracle.quant_weight(W, s)
    Y, acc, q, sx = oracle.w8a8_linear(X, s, Wq, sw, wl.act, full=True)
    sha = lambda a: hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    lines = [
        "s[:4] " + " ".join(f"{v:.9g}" for v in s[:4]),
        "sx[:4] " + " ".join(f"{v:.9g}" for v in sx[:4]),
        "sw[:4] " + " ".join(f"{v:.9g}" for v in sw[:4]),
        "q[0,:8] " + " ".join(str(int(v)) for v in q[0, :8]),
        "Wq[:8,0] " + " ".join(str(int(v)) for v in Wq[:8, 0]),
        "acc[0,:4] " + " ".join(str(int(v)) for v in acc[0, :4]),
        "Y[0,:4] " + " ".join(f"{float(v):.9g}" for v in Y[0, :4]),
        "sha256(q) " + sha(q),
        "sha256(Wq) " + sha(Wq),
        "sha256(acc) " + sha(acc),
        "sha256(Y) " + sha(Y),
    ]
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "opt125m_linear_oracle.txt")
    with open(path, "w") as f:
        f.write(compute())
    print(open(path).read())
