"""Do the pins bite?  Every entry below plants ONE plausible mistake in a copy of the oracle's C
source (a swapped index, a dropped term, a wrong sign, a transposed operand), compiles the copy and
runs the pins of tests/test_oracle_pins.py against it: at least one pin must fail for every mutant.
The mistakes are planted in the oracle only, on the CPU; every mutant keeps all accesses in bounds.
(Not in the list because it changes nothing observable here: leaving -0 unfolded in the selection --
IEEE comparison already treats -0 and +0 as equal, so the index decides either way; the fold matters
to implementations that compare bit patterns.)
"""
import itertools
import subprocess

import pytest

from oracle import oracle as vo
from tests import test_oracle_pins as pins

# (name, text in oracle/veda_oracle.c, replacement)
MUTANTS = [
    ("slots inside a tile in (h, t, w) order",
     "*l = ((t % g->pt) * g->ph + (h % g->ph)) * g->pw + (w % g->pw);",
     "*l = ((h % g->ph) * g->pt + (t % g->pt)) * g->pw + (w % g->pw);"),
    ("tiles numbered in (h, t, w) order",
     "*i = ((int64_t)(t / g->pt) * g->nh + (h / g->ph)) * g->nw + (w / g->pw);",
     "*i = ((int64_t)(h / g->ph) * g->nt + (t / g->pt)) * g->nw + (w / g->pw);"),
    ("validity bit of the wrong slot",
     "valid_mask[i * words + l / 64] |= (uint64_t)1 << (l % 64);",
     "valid_mask[i * words + l / 64] |= (uint64_t)1 << ((l ^ 1) % 64);"),
    ("channel-major tile written token-major",
     "const int64_t o = channel_major ? ((i * d + c) * B + l) : ((i * B + l) * d + c);",
     "const int64_t o = (i * B + l) * d + c;"),
    ("average over B slots instead of the real tokens",
     "const float inv = 1.0f / (float)cnt;",
     "const float inv = 1.0f / (float)(pt * ph * pw);"),
    ("max and min swapped in the descriptor",
     "zi[d + c] = mx;\n                    zi[2 * d + c] = mn;",
     "zi[d + c] = mn;\n                    zi[2 * d + c] = mx;"),
    ("descriptor sum in descending slot order",
     "for (int lt = 0; lt < pt; ++lt)\n                        for (int lh = 0; lh < ph; ++lh)\n                            for (int lw = 0; lw < pw; ++lw) {\n                                const int t = tt * pt + lt, h = th * ph + lh, w = tw * pw + lw;\n                                if (t >= T",
     "for (int lt = pt - 1; lt >= 0; --lt)\n                        for (int lh = ph - 1; lh >= 0; --lh)\n                            for (int lw = pw - 1; lw >= 0; --lw) {\n                                const int t = tt * pt + lt, h = th * ph + lh, w = tw * pw + lw;\n                                if (t >= T"),
    ("no activation between the layers",
     "hid[j] = (relu && !(acc > 0.0f)) ? 0.0f : acc;",
     "hid[j] = acc;"),
    ("first-layer weights read transposed",
     "acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * hidden + j], acc);",
     "acc = fmaf(z[r * in_dim + i], w1[(int64_t)j * in_dim + i], acc);"),
    ("second-layer bias dropped",
     "float acc = b2[o];",
     "float acc = 0.0f;"),
    ("single-layer bias dropped",
     "float acc = b1[o];",
     "float acc = 0.0f;"),
    ("first-layer chain in descending input order",
     "for (int i = 0; i < in_dim; ++i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * hidden + j], acc);",
     "for (int i = in_dim - 1; i >= 0; --i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * hidden + j], acc);"),
    ("second-layer chain in descending hidden order",
     "for (int j = 0; j < hidden; ++j) acc = fmaf(hid[j], w2[(int64_t)j * out_dim + o], acc);",
     "for (int j = hidden - 1; j >= 0; --j) acc = fmaf(hid[j], w2[(int64_t)j * out_dim + o], acc);"),
    ("single-layer chain in descending input order",
     "for (int i = 0; i < in_dim; ++i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * out_dim + o], acc);",
     "for (int i = in_dim - 1; i >= 0; --i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * out_dim + o], acc);"),
    ("score chain started from the scale instead of +0",
     "float acc = 0.0f;\n            for (int c = 0; c < dp; ++c)",
     "float acc = scale;\n            for (int c = 0; c < dp; ++c)"),
    ("score not scaled",
     "s[i * nk + j] = acc * scale;",
     "s[i * nk + j] = acc;"),
    ("score chain in descending latent order",
     "for (int c = 0; c < dp; ++c) acc = fmaf(qh[i * dp + c], kh[j * dp + c], acc);",
     "for (int c = dp - 1; c >= 0; --c) acc = fmaf(qh[i * dp + c], kh[j * dp + c], acc);"),
    ("equal scores go to the higher tile index",
     "return (x->j > y->j) - (x->j < y->j);",
     "return (x->j < y->j) - (x->j > y->j);"),
    ("the k lowest scores are kept",
     "if (x->s > y->s) return -1;\n    if (x->s < y->s) return 1;",
     "if (x->s > y->s) return 1;\n    if (x->s < y->s) return -1;"),
    ("NaN counts as +inf",
     "v = (v != v) ? -INFINITY : v + 0.0f;",
     "v = (v != v) ? INFINITY : v + 0.0f;"),
    ("kept list not put in ascending order",
     "qsort(idx + r * k, (size_t)k, sizeof(int32_t), vo_int_cmp);",
     ""),
    ("every query uses the kept list of tile 0",
     "kept[sel[(int64_t)i * ksel + t]] = 1;",
     "kept[sel[t]] = 1;"),
    ("logits not scaled",
     "a[n] = dot * scale + M[n];",
     "a[n] = dot + M[n];"),
    ("weights not normalised",
     "const double wgt = a[n] / denom;\n                ws += wgt;",
     "const double wgt = a[n];\n                ws += wgt;"),
    ("value row of the query instead of the key",
     "for (int c = 0; c < d; ++c) o[c] += wgt * (double)v[n * d + c];\n            }\n            if (lse)",
     "for (int c = 0; c < d; ++c) o[c] += wgt * (double)v[u * d + c];\n            }\n            if (lse)"),
    ("query and key swapped in the masked logit",
     "dot += (double)q[u * d + c] * (double)k[n * d + c];\n                a[n] = dot * scale + M[n];",
     "dot += (double)k[u * d + c] * (double)q[n * d + c];\n                a[n] = dot * scale + M[n];"),
    ("log-sum-exp without the subtracted maximum",
     "if (lse) lse[r] = mx + log(denom);",
     "if (lse) lse[r] = log(denom);"),
    ("dense attention not scaled",
     "a[n] = dot * scale;\n                if (a[n] > mx) mx = a[n];\n            }\n            double denom = 0.0;\n            for (int64_t n = 0; n < N; ++n) { a[n] = exp(a[n] - mx); denom += a[n]; }\n            double* o",
     "a[n] = dot;\n                if (a[n] > mx) mx = a[n];\n            }\n            double denom = 0.0;\n            for (int64_t n = 0; n < N; ++n) { a[n] = exp(a[n] - mx); denom += a[n]; }\n            double* o"),
    ("heat map pools by sum instead of maximum",
     "if (p > *cell) *cell = p;",
     "*cell += p;"),
    ("heat map of unnormalised weights",
     "const double p = a[n] / denom;\n                    double* cell",
     "const double p = a[n];\n                    double* cell"),
    ("recall counts tiles, not fractions",
     "acc += (double)common / (double)k;",
     "acc += (double)common;"),
    ("recall compares position by position",
     "if (sel_sp[i * k + a] == sel_fu[i * k + b]) { ++common; break; }",
     "if (a == b && sel_sp[i * k + a] == sel_fu[i * k + b]) { ++common; break; }"),
    ("dispersion from the sum, not the product, of the two gaps",
     "float p = up * dn;",
     "float p = up + dn;"),
    ("dispersion without the square root",
     "y[i * 2 * d + d + c] = root_lambda * sqrtf(p);",
     "y[i * 2 * d + d + c] = root_lambda * p;"),
]


def _pin_cases():
    """Every pin of tests/test_oracle_pins.py, with its parametrisations expanded."""
    out = []
    for name in sorted(vars(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn) or name == "test_planted_mistakes_are_caught_by_the_pins":
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [n.strip() for n in mark.args[0].split(",")]
            rows = [v if len(names) > 1 else (v,) for v in mark.args[1]]
            axes.append([dict(zip(names, row)) for row in rows])
        for combo in itertools.product(*axes) if axes else [()]:
            kwargs = {}
            for part in combo:
                kwargs.update(part)
            out.append((name, fn, kwargs))
    return out


def _first_failing_pin(cases):
    for name, fn, kwargs in cases:
        try:
            fn(**kwargs)
        except Exception as e:   # an assertion, or the oracle refusing its own output
            return f"{name}{kwargs or ''}: {type(e).__name__}"
    return None


@pytest.fixture
def swap_oracle():
    """Lets a test point the oracle front end at another shared library, and restores it."""
    saved = (vo._LIB, vo._lib)

    def use(path):
        vo._LIB, vo._lib = path, None
        vo.lib()

    yield use
    vo._LIB, vo._lib = saved


def test_pins_pass_on_the_oracle_itself():
    assert _first_failing_pin(_pin_cases()) is None


def test_every_planted_mistake_fails_a_pin(tmp_path, swap_oracle):
    source = vo._SRC.read_text()
    cases = _pin_cases()
    assert len(cases) >= 30
    survivors = []
    for n, (what, old, new) in enumerate(MUTANTS):
        assert source.count(old) == 1, f"mutant '{what}': its text must occur exactly once in the oracle"
        src = tmp_path / f"mutant_{n}.c"
        lib = tmp_path / f"libmutant_{n}.so"
        src.write_text(source.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-w", "-shared", "-fPIC",
                               "-o", str(lib), str(src), "-lm"])
        swap_oracle(lib)
        caught = _first_failing_pin(cases)
        print(f"mutant {n:2d} ({what}): {caught}")
        if caught is None:
            survivors.append(what)
    assert not survivors, f"no pin notices: {survivors}"
