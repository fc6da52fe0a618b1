"""Are the pins of the backward compressor's oracle sharp?  One planted mistake at a time in a copy of
oracle/naive_oracle.c; every one must fail a pin of test_naive_pins.  CPU only."""
import pytest

from oracle import build_oracle, n32
import test_naive_pins as pins
from test_oracle_mutations import _failing_pins, pins_failing_on_mutant

SRC = open(build_oracle.NAIVE_SRC).read()

MUTATIONS = [
    ("rounds half away from zero", "float r = rintf(y);", "float r = roundf(y);"),
    ("truncates", "float r = rintf(y);", "float r = truncf(y);"),
    ("upper bound 2^(b-1)", "float hi = (float)((1u << (bits - 1)) - 1u);", "float hi = (float)(1u << (bits - 1));"),
    ("symmetric lower bound", "float lo = -(float)(1u << (bits - 1));", "float lo = -(float)((1u << (bits - 1)) - 1u);"),
    ("pre-scale dropped", "float y = scale * g;", "float y = g; (void)scale;"),
    ("pre-scale not undone", "return (float)q * rc;", "(void)rc; return (float)q;"),
    ("undone by multiplying again", "float rc = 1.0f / scale;", "float rc = scale;"),
    ("no sign extension", "if (field & (1u << (b - 1))) q -= (int32_t)(1u << b);", ""),
    ("fields written most significant bit first", "if ((field >> t) & 1u) pay[", "if ((field >> (b - 1 - t)) & 1u) pay["),
    ("fields read most significant bit first", "& 1u) << t;", "& 1u) << (b - 1 - t);"),
    ("bf16 output truncated", "u += 0x7fffu + lsb;", "(void)lsb;"),
    ("bf16 input read as the low half", "<< 16;     /* bf16 widens exactly */", "<< 15;     /* bf16 widens exactly */"),
    ("width missing from the header", "hdr[5] = c->hidden; hdr[6] = c->bits;", "hdr[5] = c->hidden;"),
    ("size for whole bytes per element", "return 64 + n_elements(c) * c->bits / 8;", "return 64 + n_elements(c) * ((c->bits + 7) / 8);"),
]


def test_the_unmutated_oracle_passes_every_pin():
    assert _failing_pins(limit=1, module=pins) == []


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught_by_a_pin(what, old, new):
    assert pins_failing_on_mutant(SRC, what, old, new, n32, "NAIVE_LIB", pins), f"no pin notices: {what}"
