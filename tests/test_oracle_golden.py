"""The oracle reproduces its stored small case (written by
tests/golden/make_oracle_golden.py, which calls only oracle/)."""
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _f32(h):
    return np.frombuffer(bytes.fromhex(h), dtype=np.float32)


def load_case():
    d = json.load(open(os.path.join(HERE, "golden", "oracle_case_small.json")))
    d["off"] = np.array(d["offsets"], np.int64)
    d["grads"] = [_f32(h) for h in d["grads_f32_hex"]]
    d["tau"] = [_f32(h) for h in d["tau_f32_hex"]]
    d["s_local"] = [_f32(h) for h in d["s_local_f32_hex"]]
    d["s_shared"] = _f32(d["s_shared_f32_hex"])
    d["codes"] = [np.frombuffer(bytes.fromhex(h), dtype=np.uint8) for h in d["codes_hex"]]
    d["avg"] = _f32(d["avg_f32_hex"])
    return d


def test_oracle_reproduces_stored_case(oracle):
    d = load_case()
    for w, g in enumerate(d["grads"]):
        tau, s = oracle.clip_stats(g, d["off"], d["c"])
        assert np.array_equal(tau, d["tau"][w]) and np.array_equal(s, d["s_local"][w])
        codes = oracle.ternarize_pack(g, d["off"], tau, d["s_shared"], d["seed"], d["step"], w)
        assert np.array_equal(codes, d["codes"][w])
    assert np.array_equal(oracle.share_scalers(np.stack(d["s_local"])), d["s_shared"])
    assert np.array_equal(oracle.unpack_average(d["codes"], d["off"], d["s_shared"]), d["avg"])
