"""Writes workloads_crc.txt: CRC32 of small seeded inputs, so that a change of the generators (and
with it of every parity case and benchmark input) cannot pass unnoticed.  Calls only `workloads`.

    python tests/golden/make_workload_crcs.py
"""
import os
import sys
import zlib

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import workloads as wl  # noqa: E402


def cases():
    c = wl.config1_tiny()
    yield "config1_tiny.X", c["X"]
    yield "config1_tiny.W", c["W"]
    yield "config1_tiny.table", c["table"]
    X, t = wl.activations_persistent(2001, 64, 4096, 2)
    yield "persistent(2001,64,4096,2).X", X
    yield "persistent(2001,64,4096,2).table", t
    yield "diffuse(3003,64,512)", wl.activations_diffuse(3003, 64, 512)
    yield "weights(2100,32,4096)", wl.weights(2100, 32, 4096)
    off, rm = wl.moe_routing(4002, 256, 128, 8)
    yield "moe_routing(4002,256,128,8).offsets", off
    yield "moe_routing(4002,256,128,8).row_map", rm


if __name__ == "__main__":
    with open(os.path.join(HERE, "workloads_crc.txt"), "w") as f:
        f.write("# CRC32 of seeded generator outputs (written by make_workload_crcs.py, which calls only `workloads`)\n")
        for name, a in cases():
            f.write(f"{name} {zlib.crc32(np.ascontiguousarray(a).tobytes())}\n")
