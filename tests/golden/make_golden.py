"""Writes tests/golden/tiny_f32_oracle.json from the CPU oracle alone.

Run from the repo root:  python tests/golden/make_golden.py
The stored numbers are the oracle's float64 outputs for the small fp32 workload (inputs from
iso_inputs, seed 0).  The paper prints no numerical example, so these are not the paper's values:
they only guard the oracle and the input recipe against silent change.  Nothing here touches the
HIP path.
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import iso_inputs  # noqa: E402
from oracle import iso_oracle as orc  # noqa: E402


def main():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = orc.LayerShape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.rms_eps, wl.rope_base)
    wn = {k: iso_inputs.to_f64(v, wl.dtype) for k, v in w.items()}
    out = orc.layer_unsplit(iso_inputs.to_f64(x, wl.dtype), wn, sh)["x_out"]
    samples = [(r, c, float(out[r, c])) for r in (0, 1, 63, 64, 65, 127) for c in (0, 17, 255)]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_f32_oracle.json")
    with open(path, "w") as f:
        json.dump({"source": "oracle/iso_oracle.py layer_unsplit, workload tiny_f32, seed 0",
                   "x_out_samples": samples}, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
