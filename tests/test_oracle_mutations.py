"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a COPY of the oracle's C source
(a dropped sign, a wrong index, a transposed operand, a wrong rounding), compile it, run the pin suite
against it, and require that at least one pin fails.  Everything here runs on the CPU."""
import ctypes as C
import inspect
import os
import subprocess
import tempfile

import pytest

from oracle import build_oracle, o32
import test_oracle_pins as pins

SRC = open(build_oracle.SRC).read()

MUTATIONS = [
    ("entropy without the Shannon minus sign", "return 0.0f - invL * W;", "return invL * W;"),
    ("entropy without the common factor 1/(L1 + eps)", "return 0.0f - invL * W;", "return 0.0f - W;"),
    ("entropy of unnormalized magnitudes", "float u = fmaf(a, invL, eps_log);", "float u = a + eps_log;"),
    ("allocation tile normalised per quantization tile", "        L1 = L1 + tree_sum(w, G);\n    }\n    float invL = 1.0f / (L1 + eps_l1);\n    float W = 0.0f;\n    for (uint32_t q = 0; q < m; ++q) {\n",
     "        L1 = L1 + tree_sum(w, G);\n    }\n    float invL = 1.0f / (L1 + eps_l1);\n    float W = 0.0f;\n    for (uint32_t q = 0; q < m; ++q) {\n        for (uint32_t k = 0; k < G; ++k) w[k] = fabsf(v[q * G + k]);\n        invL = 1.0f / (tree_sum(w, G) + eps_l1);\n"),
    ("allocation tile entropy keeps only its last quantization tile", "W = W + tree_sum(w, G);", "W = tree_sum(w, G);"),
    ("allocation tile norm keeps only its last quantization tile", "L1 = L1 + tree_sum(w, G);", "L1 = tree_sum(w, G);"),
    ("k counted over quantization tiles", "double n = (double)alloc_tiles_per_unit(c);", "double n = (double)tiles_per_unit(c);"),
    ("width written to the first quantization tile of an allocation tile only",
     "for (uint32_t q = 0; q < m; ++q) width[(u * n + it[r].j) * m + q] = (uint8_t)((r < k) ? lo + 1 : lo);",
     "for (uint32_t q = 0; q < m; ++q) width[(u * n + it[r].j) * m + q] = (uint8_t)((r < k && q == 0) ? lo + 1 : lo);"),
    ("log polynomial coefficient off by 2x", "0x1.c4859ep+2f", "0x1.c4859ep+1f"),
    ("butterfly difference with swapped operands", "v[j + h] = x - y;", "v[j + h] = y - x;"),
    ("wrong 1/sqrt(G) for G = 64", "case 64: return 0.125f;", "case 64: return 0.25f;"),
    ("wrong 1/sqrt(G) for G = 8", "case 8: return 0x1.6a09e6p-2f;", "case 8: return 0x1.6a09e6p-3f;"),
    ("pivot swapped with coordinate 2 instead of 1",
     "    float t = v[0]; v[0] = v[d]; v[d] = t;\n    tahq_oracle_butterfly(v, G);\n    float c = c_G(G);",
     "    float t = v[1]; v[1] = v[d]; v[d] = t;\n    tahq_oracle_butterfly(v, G);\n    float c = c_G(G);"),
    ("inverse transform forgets to undo the swap",
     "    for (uint32_t k = 0; k < G; ++k) v[k] = v[k] * c;\n    float t = v[0]; v[0] = v[d]; v[d] = t;\n}",
     "    for (uint32_t k = 0; k < G; ++k) v[k] = v[k] * c;\n    (void)d;\n}"),
    ("outlier test not strict", "return a1 > t2;", "return a1 >= t2;"),
    ("argmax tie goes to the last index", "if (fabsf(v[k]) > a1) { a1 = fabsf(v[k]); d = k; }",
     "if (fabsf(v[k]) >= a1) { a1 = fabsf(v[k]); d = k; }"),
    ("second largest ignores multiplicity", "if (k != d && fabsf(v[k]) > a2) a2 = fabsf(v[k]);",
     "if (fabsf(v[k]) != a1 && fabsf(v[k]) > a2) a2 = fabsf(v[k]);"),
    ("allocation ties go to the higher index", "return (a->j > b->j) - (a->j < b->j);",
     "return (a->j < b->j) - (a->j > b->j);"),
    ("allocation picks the lowest entropies", "if (a->H > b->H) return -1;\n    if (a->H < b->H) return 1;",
     "if (a->H > b->H) return 1;\n    if (a->H < b->H) return -1;"),
    ("k truncated instead of rounded", "* n + 0.5);", "* n);"),
    ("quantizer rounds half up", "rintf(t)", "floorf(t + 0.5f)"),
    ("quantizer uses 2^b steps", "float Lv = (float)((1u << b) - 1u);\n    uint16_t z", "float Lv = (float)(1u << b);\n    uint16_t z"),
    ("k counted from three bits whatever the low width", "- (double)low_bits(c) * n + 0.5);", "- 3.0 * n + 0.5);"),
    # (planted mistakes must keep the mutant inside its buffers: it runs in this process)
    ("zero-point rounded to nearest instead of down",
     "if (tahq_oracle_fp16_widen(h) > xc) h = fp16_prev(h);", ""),
    ("scale rounded to nearest instead of up",
     "if (tahq_oracle_fp16_widen(h) < xc) h = fp16_next(h);", ""),
    ("payload elements in reverse order", "uint32_t bit = b * k;\n            /* a code spans", "uint32_t bit = b * (G - 1 - k);\n            /* a code spans"),
    ("rank table off by one", "put_u32(packed + L.ranks + 4 * (j >> 6), (uint32_t)rank);",
     "put_u32(packed + L.ranks + 4 * (j >> 6), (uint32_t)rank + 1);"),
    ("bit map marks three-bit tiles", "if (b == lo + 1) packed[L.bitmap + (j >> 3)] |=", "if (b == lo) packed[L.bitmap + (j >> 3)] |="),
    ("de-quantization without the zero-point", "return fmaf((float)q, tahq_oracle_fp16_widen(s16), tahq_oracle_fp16_widen(z16));",
     "(void)z16; return (float)q * tahq_oracle_fp16_widen(s16);"),
    ("bf16 narrowing truncates", "u += 0x7fffu + lsb;", "(void)lsb;"),
    ("range taken before the transform",
     "    for (uint32_t k = 0; k < G; ++k) y[k] = v[k];\n    if (flag) tahq_oracle_forward_transform(y, G, d);\n    float mn = y[0], mx = y[0];\n    for (uint32_t k = 1; k < G; ++k) { mn = fminf(mn, y[k]); mx = fmaxf(mx, y[k]); }",
     "    for (uint32_t k = 0; k < G; ++k) y[k] = v[k];\n    float mn = y[0], mx = y[0];\n    for (uint32_t k = 1; k < G; ++k) { mn = fminf(mn, y[k]); mx = fmaxf(mx, y[k]); }\n    if (flag) tahq_oracle_forward_transform(y, G, d);"),
]


def _pin_calls(module=pins):
    """Every pin of a test module as a list of zero-argument callables (parametrized ones expanded)."""
    calls = []
    for name, fn in sorted(vars(module).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        combos = [{}]
        for m in marks:
            names = [s.strip() for s in m.args[0].split(",")]
            new = []
            for base in combos:
                for val in m.args[1]:
                    vals = val if len(names) > 1 else (val,)
                    d = dict(base)
                    d.update(zip(names, vals))
                    new.append(d)
            combos = new
        for kw in combos:
            calls.append((f"{name}{kw}", lambda fn=fn, kw=kw: fn(**kw)))
    return calls


def _failing_pins(limit=1, module=pins):
    failed = []
    for name, call in _pin_calls(module):
        try:
            call()
        except AssertionError:
            failed.append(name)
        except Exception as e:            # a mutated oracle may also trip an index or value error in a pin
            failed.append(f"{name} ({type(e).__name__})")
        if len(failed) >= limit:
            break
    return failed


def test_the_unmutated_oracle_passes_every_pin():
    assert _failing_pins(limit=1) == []


def pins_failing_on_mutant(source, what, old, new, wrapper, lib_attr, module):
    """Compile `source` with `old` replaced by `new`, point the ctypes wrapper at it, run the pins of `module`."""
    assert source.count(old) == 1, f"mutation anchor for '{what}' must match the oracle source exactly once"
    saved = wrapper._lib
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "mutant.c")
        lib = os.path.join(tmp, "libmutant.so")
        open(src, "w").write(source.replace(old, new))
        flags = [f for f in build_oracle.CFLAGS if f != "-Werror"]
        subprocess.run(["gcc"] + flags + [src, "-o", lib, "-lm"], check=True)
        try:
            wrapper._lib = None
            orig = getattr(build_oracle, lib_attr)
            setattr(build_oracle, lib_attr, lib)
            try:
                wrapper.lib()
            finally:
                setattr(build_oracle, lib_attr, orig)
            failed = _failing_pins(limit=1, module=module)
        finally:
            wrapper._lib = saved
    return failed


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught_by_a_pin(what, old, new):
    assert pins_failing_on_mutant(SRC, what, old, new, o32, "LIB", pins), f"no pin notices: {what}"
