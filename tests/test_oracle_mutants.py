"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a dropped term, a wrong sign or index, a transposed operand, an off-by-one), builds it, and runs
the pins of tests/test_oracle_pins.py against the mutant: at least one pin has to fail.

CPU only; the mistakes live in a temporary copy of the oracle, never in the HIP path.
"""
import ctypes
import inspect
import subprocess

import pytest

from oracle import less_oracle as lo
from tests import test_oracle_pins as pins

SRC = (lo._HERE / "less_oracle.c").read_text()

# (name, text in the oracle, what a mistaken author might have written)
MUTANTS = [
    ("denominator-without-low-rank-term", "    double den = wl;", "    double den = 0.0;"),
    ("numerator-without-low-rank-term", "        og[d] = a * sh;", "        og[d] = 0.0 * a * sh;"),
    ("score-sign", "      sc[j] = a / sqrtD;", "      sc[j] = -a / sqrtD;"),
    ("score-scale-D-instead-of-sqrt-D", "  const double sqrtD = sqrt((double)D);\n  int rc = 0;",
     "  const double sqrtD = (double)D;\n  int rc = 0;"),
    ("phi-first-matrix-transposed", "    for (int d = 0; d < D; ++d) a += q[d] * W1[(size_t)d * Rp + i];",
     "    for (int d = 0; d < D; ++d) a += q[d] * W1[(size_t)i * D + d];"),
    ("psi-third-matrix-transposed", "    for (int i = 0; i < R; ++i) a += h2[i] * W3[(size_t)i * R + r];",
     "    for (int i = 0; i < R; ++i) a += h2[i] * W3[(size_t)r * R + i];"),
    ("psi-without-absolute-value", "    g[r] = fabs(a);", "    g[r] = a;"),
    ("phi-without-absolute-value", "    f[r] = fabs(less_oracle_gelu(a));", "    f[r] = less_oracle_gelu(a);"),
    ("gelu-argument-scale", "return 0.5 * x * erfc(-x / sqrt(2.0));", "return 0.5 * x * erfc(-x);"),
    ("new-token-starts-with-zero-score", "  double acc_new = inc[C];", "  double acc_new = 0.0 * inc[C];"),
    ("scores-not-accumulated", "    if (s->pos[j] >= 0) s->acc[j] += inc[j];",
     "    if (s->pos[j] >= 0) s->acc[j] = inc[j];"),
    ("only-the-first-query-head-scores", "      if (s->pos[j] >= 0) inc[j] += e[j] / dacc;",
     "      if (s->pos[j] >= 0 && g == 0) inc[j] += e[j] / dacc;"),
    ("query-heads-share-the-first-phi",
     "    less_oracle_phi(qg, s->Wq1 + (size_t)g * D * s->Rp, s->Wq2 + (size_t)g * s->Rp * R, D, s->Rp, R, f);   /* Eq. 1 */",
     "    less_oracle_phi(qg, s->Wq1, s->Wq2, D, s->Rp, R, f);"),
    ("prompt-scores-from-the-last-query-head-only",
     "      for (int64_t j = 0; j <= i; ++j) { row[j] /= L; colsum[j] += row[j]; }",
     "      for (int64_t j = 0; j <= i; ++j) { row[j] /= L; if (g == s->G - 1) colsum[j] += row[j]; }"),
    ("recent-window-off-by-one", "      else { if (s->pos[j] > n - s->Nr) continue;",
     "      else { if (s->pos[j] >= n - s->Nr) continue;"),
    ("evicts-the-largest-score", "      if (a < bacc || (a == bacc && p < bpos)) {",
     "      if (a > bacc || bpos < 0 || (a == bacc && p < bpos)) {"),
    ("tie-evicts-the-newer-token", "      if (a < bacc || (a == bacc && p < bpos)) {",
     "      if (a < bacc || (a == bacc && p > bpos)) {"),
    ("z-not-updated", "    s->z[r] += g[r];", "    s->z[r] += 0.0 * g[r];"),
    ("H-updated-with-key-instead-of-value",
     "    for (int d = 0; d < s->D; ++d) s->H[(size_t)r * s->D + d] += g[r] * v[d];",
     "    for (int d = 0; d < s->D; ++d) s->H[(size_t)r * s->D + d] += g[r] * k[d];"),
    ("state-folded-before-the-output",      # Algorithm 1 uses H_t, z_t from before this step's eviction
     "  double share_sum = 0.0;\n",
     "  double share_sum = 0.0;\n"
     "  if (n >= C && C > 0 && s->Nr > 0) { int jm = 0; for (int j = 1; j < C; ++j) if (s->pos[j] < s->pos[jm]) jm = j;\n"
     "    double gg[64]; less_oracle_psi(s->Kc + (size_t)jm * D, s->Wk1, s->Wk2, s->Wk3, D, s->Rp, R, gg);\n"
     "    for (int r = 0; r < R; ++r) s->z[r] += 1e-3 * gg[r]; }"),
    ("prompt-keeps-the-smallest-column-sums", "  if (a->a < b->a) return -1;\n  if (a->a > b->a) return 1;",
     "  if (a->a < b->a) return 1;\n  if (a->a > b->a) return -1;"),
    ("prompt-column-sums-unnormalised", "      for (int64_t j = 0; j <= i; ++j) { row[j] /= L; colsum[j] += row[j]; }",
     "      for (int64_t j = 0; j <= i; ++j) { colsum[j] += row[j]; row[j] /= L; }"),
    ("prompt-recent-window-off-by-one", "    int64_t ncand = P - s->Nr;                            /* positions < P - Nr */",
     "    int64_t ncand = P - s->Nr + 1;"),
    ("prompt-discarded-pairs-not-folded", "      fold_into_state(s, K + j * D, V + j * D);           /* Eq. 6 */",
     "      (void)0;"),
    ("lambda-first-tokens-not-protected", "        if (j >= 0 && p < s->Nh) continue;", "        (void)0;"),
    ("lambda-prompt-keeps-heavy-hitters", "  } else if (s->flags & LESS_FLAG_LAMBDA) {", "  } else if (0) {"),
    ("budget-rounded-to-nearest", "floor(tokens / 2.0 + 1e-9)", "floor(tokens / 2.0 + 0.5)"),
    ("sparse-denominator-flag-ignored", "(s->flags & LESS_FLAG_SPARSE_DENOM) ? (den - wl) : den", "den"),
    ("hellinger-without-square-roots", "double d = sqrt(p[i]) - sqrt(q[i]);", "double d = p[i] - q[i];"),
]


def _pin_calls():
    """Every pin as a zero-argument callable (parametrized ones once per parameter set)."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        argnames, values = marks[0].args
        names = [a.strip() for a in argnames.split(",")]
        for v in values:
            v = v if isinstance(v, (tuple, list)) else (v,)
            calls.append((f"{name}{list(v)}", (lambda f=fn, kw=dict(zip(names, v)): f(**kw))))
    return calls


@pytest.fixture()
def restore_oracle():
    yield
    lo._lib = None
    lo.lib()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(name, old, new, tmp_path, restore_oracle):
    assert SRC.count(old) == 1, f"mutation site of {name} not found exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(SRC.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(src), "-lm"])
    good = lo.lib()
    mutant = ctypes.CDLL(str(so))
    for fn in ("less_oracle_budget_tokens", "less_oracle_gelu", "less_oracle_hellinger", "less_oracle_phi",
               "less_oracle_psi", "less_oracle_reset", "less_oracle_step", "less_oracle_prefill"):
        getattr(mutant, fn).restype = getattr(good, fn).restype
        getattr(mutant, fn).argtypes = getattr(good, fn).argtypes
    lo._lib = mutant
    killed_by = []
    for pin_name, call in _pin_calls():
        try:
            call()
        except Exception:                       # an assertion, or the mutant's own breakage
            killed_by.append(pin_name)
    print(f"{name}: caught by {len(killed_by)} pins: {', '.join(killed_by)}")
    assert killed_by, f"no pin notices: {name}"
