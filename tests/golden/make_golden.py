"""Writes tests/golden/oracle_digests.json: SHA-256 of the CPU oracle's int8 output on
reduced-batch versions of the five benchmark workloads.

Calls only ``oracle`` and the seeded input generators.  The digests guard the oracle against
accidental change; they are not an independent source of truth (the pins in test_oracle_*.py are).

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import BASELINE_CONFIGS as CONFIG_ORDER, make_workload  # noqa: E402

BATCH = {"deit_tiny_b1": 1, "vit_b16_b64": 2, "deit_b384_b32": 1, "swin_t_s1_b64": 128,
         "vit_l384_heavy": 1}


def digests():
    out = {}
    for name in CONFIG_ORDER:
        wl = make_workload(name, batch=BATCH[name])
        p = oracle.derive_params(wl.sQ, wl.sK, wl.shape[-1])
        for tile in wl.kv_tiles:
            o = oracle.qflash_attention(wl.Q, wl.K, wl.V, p, tile, bias=wl.bias)
            out["%s/b%d/kv%d" % (name, BATCH[name], tile)] = {
                "params": list(p.astuple()),
                "inputs_sha256": hashlib.sha256(
                    wl.Q.tobytes() + wl.K.tobytes() + wl.V.tobytes()).hexdigest(),
                "output_sha256": hashlib.sha256(o.tobytes()).hexdigest(),
            }
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digests.json")
    with open(path, "w") as f:
        json.dump(digests(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
