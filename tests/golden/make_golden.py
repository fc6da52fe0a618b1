"""Writes tests/golden/oracle_streams.sha256.txt: SHA-256 of the streams and decoded tensors that the CPU
oracles produce on small seeded workloads.  Calls only oracle/ and the seeded generators; the stored
digests pin the oracles against accidental change (a deliberate change to their arithmetic re-runs this
script and says why in its commit message).

    python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads                       # noqa: E402
from oracle import n32, o32            # noqa: E402

OUT = os.path.join(HERE, "oracle_streams.sha256.txt")

# (name, workload index, generator shape, oracle configuration keywords)
FORWARD = [
    ("cfg1_default", 1, dict(batch=1, seq=16), dict()),
    ("cfg2_default", 2, dict(batch=2, seq=24), dict()),
    ("cfg3_default", 3, dict(batch=2, seq=8), dict()),
    ("cfg4_default", 4, dict(batch=2, seq=40), dict()),
    ("cfg5_default", 5, dict(batch=2, seq=16), dict()),
    ("cfg4_budget3.8", 4, dict(batch=2, seq=40), dict(budget_bits=3.8)),
    ("cfg2_scope1_tau4", 2, dict(batch=2, seq=24), dict(scope=1, tau=4.0)),
    ("cfg4_token_level", 4, dict(batch=2, seq=10), dict(alloc_tile=8192)),
    ("cfg4_int2_int3", 4, dict(batch=2, seq=40), dict(budget_bits=2.2, low_bits=2)),
    ("cfg4_tile8", 4, dict(batch=1, seq=6), dict(tile=8)),
    ("cfg2_tile16", 2, dict(batch=1, seq=12), dict(tile=16)),
]
BACKWARD = [
    ("cfg5_8bit", 5, dict(batch=2, seq=16), dict(bits=8, scale=2.0 ** 14)),
    ("cfg5_6bit", 5, dict(batch=2, seq=16), dict(bits=6, scale=2.0 ** 12)),
    ("cfg2_10bit", 2, dict(batch=1, seq=24), dict(bits=10, scale=100.0)),
    ("cfg5_4bit", 5, dict(batch=1, seq=16), dict(bits=4, scale=2.0 ** 9)),
]


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def forward_case(index, shape, kw):
    w, x = workloads.generate(index, **shape)
    kw = dict(kw)
    cfg = o32.make_cfg(w.batch, w.seq, w.hidden, kw.pop("tile", w.tile), w.dtype, kw.pop("budget_bits", w.budget_bits), **kw)
    packed = o32.encode(cfg, x)
    return digest(packed), digest(o32.decode(cfg, packed, o32.F32)), digest(o32.decode(cfg, packed, o32.BF16))


def backward_case(index, shape, kw):
    w, x = workloads.generate(index, **shape)
    cfg = n32.make_cfg(w.batch, w.seq, w.hidden, w.dtype, kw["bits"], kw["scale"])
    packed = n32.encode(cfg, x)
    return digest(packed), digest(n32.decode(cfg, packed, n32.F32)), digest(n32.decode(cfg, packed, n32.BF16))


def lines():
    yield "# written by tests/golden/make_golden.py from the CPU oracles; columns: case, stream, fp32 decode, bf16 decode"
    for name, index, shape, kw in FORWARD:
        yield " ".join(("forward/" + name,) + forward_case(index, shape, kw))
    for name, index, shape, kw in BACKWARD:
        yield " ".join(("backward/" + name,) + backward_case(index, shape, kw))


if __name__ == "__main__":
    with open(OUT, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print(OUT)
