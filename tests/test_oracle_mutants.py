"""The pins must notice plausible mistakes.  Each case below plants one mistake in a copy of the
oracle's C source (on the CPU, in a temporary directory), compiles it and runs the pin checks
of test_oracle_pins against the mutant: at least one of them has to fail."""
import os

import pytest

import oracle
from oracle import lnmod_oracle
from test_oracle_pins import PIN_FUNCS

# (label, text to find, replacement, which occurrence: 0-based index or "all")
MUTANTS = [
    ("mean divides by D-1", "double mu = s / (double)D;", "double mu = s / (double)(D - 1);", 0),
    ("unbiased variance", "double var = q / (double)D;", "double var = q / (double)(D - 1);", 0),
    ("eps outside the sqrt", "1.0 / sqrt(var + eps)", "1.0 / (sqrt(var) + eps)", 0),
    ("eps dropped", "1.0 / sqrt(var + eps)", "1.0 / sqrt(var)", 0),
    ("variance not centred", "double c = ld(x, in_f32, row * D + d) - mu;",
     "double c = ld(x, in_f32, row * D + d);", 0),
    ("forward: scale instead of 1+scale", "xhat * (1.0 + ld(scale", "xhat * (ld(scale", 0),
    ("forward: shift subtracted", "+ ld(shift, in_f32, mrow * D + d);", "- ld(shift, in_f32, mrow * D + d);", 0),
    ("forward: wrong modulation row", "(mod == LNMOD_ORACLE_PER_TOKEN) ? n : m;",
     "(mod == LNMOD_ORACLE_PER_TOKEN) ? n : 0;", 0),
    ("backward: wrong modulation row", "(mod == LNMOD_ORACLE_PER_TOKEN) ? n : m;",
     "(mod == LNMOD_ORACLE_PER_TOKEN) ? n : 0;", 1),
    ("forward: rstd saved as std", "rstd[n] = r;", "rstd[n] = 1.0 / r;", 0),
    ("backward: g without 1+scale (reductions)",
     "double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, mrow * D + d));",
     "double g = ld(dy, in_f32, n * D + d);", 0),
    ("backward: g without 1+scale (dx)",
     "double g = ld(dy, in_f32, n * D + d) * (1.0 + ld(scale, in_f32, mrow * D + d));",
     "double g = ld(dy, in_f32, n * D + d);", 1),
    ("backward: c2 sums g only", "s2 += g * xhat;", "s2 += g;", 0),
    ("backward: c1 term dropped", "r[n] * (g - c1 - xhat * c2)", "r[n] * (g - xhat * c2)", 0),
    ("backward: c2 term sign", "r[n] * (g - c1 - xhat * c2)", "r[n] * (g - c1 + xhat * c2)", 0),
    ("backward: c2 term dropped", "r[n] * (g - c1 - xhat * c2)", "r[n] * (g - c1)", 0),
    ("backward: dx not scaled by rstd", "r[n] * (g - c1 - xhat * c2)", "(g - c1 - xhat * c2)", 0),
    ("backward: per-token dscale without xhat",
     "dscale[n * D + d] = ld(dy, in_f32, n * D + d) * xhat;",
     "dscale[n * D + d] = ld(dy, in_f32, n * D + d);", 0),
    ("backward: per-token dshift takes g", "dshift[n * D + d] = ld(dy, in_f32, n * D + d);",
     "dshift[n * D + d] = g;", 0),
    ("backward: dscale sums dy only", "dscale[m * D + d] += t * xhat;", "dscale[m * D + d] += t;", 0),
    ("backward: dshift sums dy*xhat", "dshift[m * D + d] += t;", "dshift[m * D + d] += t * xhat;", 0),
    ("backward: token sum skips the last token", "for (int64_t n = n0; n < n1; ++n) {\n                    for",
     "for (int64_t n = n0; n < n1 - 1; ++n) {\n                    for", 0),
    ("backward: xhat without rstd in sums",
     "double xhat = (ld(x, in_f32, n * D + d) - mu[n]) * r[n];",
     "double xhat = (ld(x, in_f32, n * D + d) - mu[n]);", 2),
]


def _replace_nth(text, old, new, nth):
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(old, pos + 1)
        if pos < 0:
            raise AssertionError("mutation site not found: %r (occurrence %d)" % (old, nth))
    return text[:pos] + new + text[pos + len(old):]


@pytest.mark.parametrize("label,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, label, old, new, nth):
    with open(lnmod_oracle.SOURCE) as f:
        src = f.read()
    mutated = _replace_nth(src, old, new, nth)
    assert mutated != src
    c_path = os.path.join(tmp_path, "mutant.c")
    with open(c_path, "w") as f:
        f.write(mutated)
    so_path = oracle.build(force=True, source=c_path, output=os.path.join(tmp_path, "libmutant.so"))
    lib = oracle.load(so_path)
    caught = []
    for check in PIN_FUNCS:
        try:
            check(lib)
        except AssertionError:
            caught.append(check.__name__)
    assert caught, "no pin notices the planted mistake: " + label


def test_unmutated_source_passes_every_pin(tmp_path):
    so_path = oracle.build(force=True, source=lnmod_oracle.SOURCE,
                           output=os.path.join(tmp_path, "libclean.so"))
    lib = oracle.load(so_path)
    for check in PIN_FUNCS:
        check(lib)
