"""Writes oracle_c1_reference.json from the CPU oracle alone (no GPU code is imported or called)."""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import dp_synth as syn  # noqa: E402
from oracle import dp_oracle as orc  # noqa: E402


def build():
    cfg = syn.CONFIGS["C1"]
    B, T, C = cfg["B"], cfg["T"], cfg["C"]
    A = syn.normal_f32((B, T, 64), cfg["act_std"], cfg["data_seed"])
    G = syn.normal_f32((B, T, 64), cfg["grad_std"], cfg["data_seed"] + 1)
    W = syn.normal_f32((64 * 64,), 0.02, cfg["data_seed"] + 2)
    n = orc.sqnorms_dense(A, G, False)
    c = orc.clip_factors(n, C)
    S, _ = orc.clip_accumulate_dense(A, G, c, False)
    kw = dict(elem_offset=0, C=C, seed=0, step=1, batch_size=B, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-11, weight_decay=0.01)
    th0, m0, v0, _ = orc.noise_adamw(W, np.zeros(4096), np.zeros(4096), S.reshape(-1).astype(np.float32), sigma=0.0, **kw)
    th1, m1, v1, _ = orc.noise_adamw(W, np.zeros(4096), np.zeros(4096), S.reshape(-1).astype(np.float32), sigma=1.0, **kw)
    idx = [0, 1, 63, 64, 2047, 4095]
    return dict(
        sqnorms=[float(x) for x in n], clip=[float(x) for x in c],
        sum_idx=idx, sum=[float(S.reshape(-1)[i]) for i in idx],
        theta_sigma0=[float(th0[i]) for i in idx], m_sigma1=[float(m1[i]) for i in idx],
        theta_sigma1=[float(th1[i]) for i in idx],
        philox_seed0_step1=[int(x) for x in orc.philox_u32(8, 0, 0, 1)],
        philox_seed1234_step1=[int(x) for x in orc.philox_u32(8, 0, 1234, 1)],
        normals_seed1234_step1=[float(x) for x in orc.normals(8, 0, 1234, 1)],
    )


if __name__ == "__main__":
    with open(os.path.join(HERE, "oracle_c1_reference.json"), "w") as f:
        json.dump(build(), f, indent=1)
    print("written")
