"""The hand-written file of tests/golden/two_tensor_file.txt against the oracle and against the
library's planner (header only; the planner needs no GPU)."""
import os

import numpy as np

from oracle import oracle
from paper_2406_10707_amd import binding as B
from paper_2406_10707_amd import shards

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    size, parts = None, []
    for line in open(os.path.join(HERE, "golden", "two_tensor_file.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, val = line.split(":")
        if key == "size":
            size = int(val, 16)
        else:
            parts.append((int(key, 16), bytes.fromhex(val.replace(" ", ""))))
    blob = bytearray(size)
    for off, b in parts:
        assert not any(blob[off:off + len(b)])
        blob[off:off + len(b)] = b
    return bytes(blob)


def test_oracle_writes_the_hand_made_file():
    w = np.array([1, 2, 3, 4, 5, 6], dtype=np.uint8)
    b = np.array([0xAA, 0xBB, 0xCC, 0xDD], dtype=np.uint8)
    tensors = [("w", shards.BF16, (3,), w), ("b", shards.F32, (), b)]
    assert oracle.serialize_bytes(tensors, 7) == _golden()


def test_planner_header_is_the_hand_made_header():
    plan = B.Plan([("w", B.CKPT_BF16, (3,), 0x7000_0000_0000, 6), ("b", B.CKPT_F32, (), 0x7000_0000_1000, 4)])
    assert plan.header(7) == _golden()[:4096]
    assert plan.offsets() == [4096, 8192] and plan.layout()["file_bytes"] == 0x3000
    plan.close()
