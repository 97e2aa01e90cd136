"""Writes tests/golden/oracle_case_small.json: a small fixed input and what the
CPU oracle computes for it.  Calls only `oracle/`; run from the repo root:
    python tests/golden/make_oracle_golden.py
The stored values guard the oracle's arithmetic against accidental change; a
deliberate change of a reading regenerates this file in the same commit.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def main():
    rng = np.random.default_rng(20170523)
    sizes = [5, 20, 1, 0, 37, 64, 3]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n, W, c = int(off[-1]), 3, 2.5
    sig = [1e-2, 3e-4, 1.0, 1.0, 2e-3, 5e-3, 1e-4]
    grads = []
    for w in range(W):
        g = np.concatenate([rng.normal(size=s) * sg for s, sg in zip(sizes, sig)]).astype(np.float32)
        g[rng.integers(0, n, size=3)] *= 25.0
        grads.append(g)
    taus, s_loc = zip(*[oracle.clip_stats(g, off, c) for g in grads])
    s_shared = oracle.share_scalers(np.stack(s_loc))
    seed, step = 0xC0FFEE123456789, 17
    codes = [oracle.ternarize_pack(g, off, t, s_shared, seed, step, w) for w, (g, t) in enumerate(zip(grads, taus))]
    avg = oracle.unpack_average(codes, off, s_shared)
    out = {
        "offsets": off.tolist(), "n_workers": W, "c": c, "seed": seed, "step": step,
        "grads_f32_hex": [g.tobytes().hex() for g in grads],
        "tau_f32_hex": [np.asarray(t, np.float32).tobytes().hex() for t in taus],
        "s_local_f32_hex": [np.asarray(s, np.float32).tobytes().hex() for s in s_loc],
        "s_shared_f32_hex": s_shared.tobytes().hex(),
        "codes_hex": [cd.tobytes().hex() for cd in codes],
        "avg_f32_hex": avg.tobytes().hex(),
    }
    with open(os.path.join(HERE, "oracle_case_small.json"), "w") as f:
        json.dump(out, f, indent=0)
    print("wrote oracle_case_small.json: n=%d W=%d" % (n, W))


if __name__ == "__main__":
    main()
