"""Writes tests/golden/config1_oracle.txt from the CPU oracle alone (never from the HIP path).

Run from the repo root:  python -m tests.golden.make_golden
"""
import hashlib
import os

import numpy as np

import oracle
import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def config1_digest() -> str:
    s = synth.layer_spec(1)
    X, W, u = synth.make_activation_frames(s), synth.make_weights(s), synth.make_signs(s)
    a = oracle.rotated_col_absmax(X, pre_signs=u)
    prep = oracle.prepare_weights(W, a, pre_signs=u, alpha=0.5)
    res = oracle.linear(X, prep, pre_signs=u)
    lines = [
        "# oracle digest of config 1 (tiny W4A4 linear, seed 0); regenerate with python -m tests.golden.make_golden",
        "qx_sha256 " + hashlib.sha256(np.ascontiguousarray(res.qx).tobytes()).hexdigest(),
        "qw_sha256 " + hashlib.sha256(np.ascontiguousarray(prep.qw).tobytes()).hexdigest(),
        "acc_sha256 " + hashlib.sha256(np.ascontiguousarray(res.acc).tobytes()).hexdigest(),
        "Y_sha256 " + hashlib.sha256(np.ascontiguousarray(res.Y).tobytes()).hexdigest(),
        "acc[0,:8] " + " ".join(str(int(v)) for v in res.acc[0, :8]),
        "Y[0,:8] " + " ".join(f"{int(v):04x}" for v in res.Y[0, :8]),
        "dx[:4] " + " ".join(float(v).hex() for v in res.dx[:4]),
        "dw[:4] " + " ".join(float(v).hex() for v in prep.dw[:4]),
    ]
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(os.path.join(HERE, "config1_oracle.txt"), "w") as f:
        f.write(config1_digest())
    print(config1_digest())
