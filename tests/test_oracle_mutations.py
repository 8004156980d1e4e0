"""Planted mistakes in the CPU oracle: each one is compiled from a temporary copy of oracle/jfa_oracle.c and must be
caught by at least one pin of tests/test_oracle_pins.py.  This is what shows that the pins constrain every term of
the oracle (paper Section 2.1: scores, row softmax with its maximum, second product; Section 2.2: the gradients)."""
import os

import pytest

import oracle_variants as ov
import test_oracle_pins as pins

# (what is planted, text in jfa_oracle.c, its replacement)
MUTATIONS = [
    ("scores not scaled by 1/sqrt(D)", "S[i * L + j] = acc * inv_sqrt_d;", "S[i * L + j] = acc;"),
    ("row maximum not subtracted", "double mi = S[i * L];", "double mi = 0.0;"),
    ("lse without the maximum", "= m[i] + log(l[i]);", "= log(l[i]);"),
    ("lse in base 2", "= m[i] + log(l[i]);", "= m[i] + log2(l[i]);"),
    ("P transposed in the second product", "o[d] += S[i * L + j] * (double)v[at(s + j, h, d, H, D)];",
     "o[d] += S[j * L + i] * (double)v[at(s + j, h, d, H, D)];"),
    ("dS with delta added", "const double ds = p * (dp - dl[i]);", "const double ds = p * (dp + dl[i]);"),
    ("dS without delta", "const double ds = p * (dp - dl[i]);", "const double ds = p * (dp);"),
    ("delta of the key instead of the query", "const double ds = p * (dp - dl[i]);", "const double ds = p * (dp - dl[j]);"),
    ("dV with query and key swapped", "dv[at(s + j, h, d, H, D)] += p * (double)dout[at(s + i, h, d, H, D)];",
     "dv[at(s + i, h, d, H, D)] += p * (double)dout[at(s + j, h, d, H, D)];"),
    ("dQ not scaled", "dq[at(s + i, h, d, H, D)] *= inv_sqrt_d;", "dq[at(s + i, h, d, H, D)] *= 1.0;"),
    ("dK not scaled", "dk[at(s + i, h, d, H, D)] *= inv_sqrt_d;", "dk[at(s + i, h, d, H, D)] *= 1.0;"),
    ("dK from the key's own query row", "dk[at(s + j, h, d, H, D)] += ds * (double)q[at(s + i, h, d, H, D)];",
     "dk[at(s + j, h, d, H, D)] += ds * (double)q[at(s + j, h, d, H, D)];"),
    ("dQ from Q instead of K", "dq[at(s + i, h, d, H, D)] += ds * (double)k[at(s + j, h, d, H, D)];",
     "dq[at(s + i, h, d, H, D)] += ds * (double)q[at(s + j, h, d, H, D)];"),
    ("dP from K instead of V", "dp += (double)dout[at(s + i, h, d, H, D)] * (double)v[at(s + j, h, d, H, D)];",
     "dp += (double)dout[at(s + i, h, d, H, D)] * (double)k[at(s + j, h, d, H, D)];"),
    ("keys always taken from head 0", "acc += (double)q[at(s + i, h, d, H, D)] * (double)k[at(s + j, h, d, H, D)];",
     "acc += (double)q[at(s + i, h, d, H, D)] * (double)k[at(s + j, 0, d, H, D)];"),
    ("values always taken from head 0", "o[d] += S[i * L + j] * (double)v[at(s + j, h, d, H, D)];",
     "o[d] += S[i * L + j] * (double)v[at(s + j, 0, d, H, D)];"),
    ("softmax not normalised", "S[i * L + j] = exp(S[i * L + j] - m[i]) / l[i];", "S[i * L + j] = exp(S[i * L + j] - m[i]);"),
]


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, what, old, new):
    text = open(ov.ORACLE_SRC).read()
    assert text.count(old) >= 1, f"the oracle no longer contains the line this mutation edits: {old}"
    src = tmp_path / "jfa_oracle_mutant.c"
    src.write_text(text.replace(old, new, 1))
    mutant = ov.oracle_module_for(ov.compile_oracle(str(src), str(tmp_path / "libmutant.so")))
    for name, call in ov.pin_calls(pins):
        try:
            call(mutant)
        except Exception:   # an assertion of the pin, or an error raised on the way to it
            return
    pytest.fail(f"no pin notices: {what}")


def test_the_unmodified_oracle_passes_the_same_calls(tmp_path):
    """The harness above, applied to an exact copy: every pin call must pass (so a failure there means a mistake)."""
    src = tmp_path / "jfa_oracle_copy.c"
    src.write_text(open(ov.ORACLE_SRC).read())
    copy = ov.oracle_module_for(ov.compile_oracle(str(src), str(tmp_path / "libcopy.so")))
    calls = ov.pin_calls(pins)
    assert len(calls) >= 15
    for name, call in calls:
        call(copy)
