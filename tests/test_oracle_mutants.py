"""Do the oracle's pins notice a mistake?  CPU only.

Each entry below plants one plausible mistake in a copy of oracle/sfi_oracle.c (a dropped term, a wrong sign,
index, edge or exponent, a missing epsilon or clamp), builds the copy in a temporary directory and runs the
pin tests against it (SFI_ORACLE_LIB points the oracle's loader at the copy).  Every one of them has to fail.
The stored-values test (test_oracle_golden.py) is left out on purpose: it is the oracle's own output and
pins nothing.  The unchanged source, built the same way, has to pass.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "sfi_oracle.c")
PIN_FILES = ["test_oracle_attention.py", "test_oracle_selector.py", "test_oracle_trigger.py",
             "test_oracle_window.py", "test_oracle_loop.py"]

# (name, text in the source, replacement).  The text must occur exactly once.
MUTANTS = [
    # allowed set, index sets, GQA mapping
    ("J upper edge", "const int64_t j_hi = L - c->recent;", "const int64_t j_hi = L - c->recent + 1;"),
    ("J lower edge", "const int64_t j_lo = c->n_sink; ", "const int64_t j_lo = c->n_sink + 1; "),
    ("GQA map of dense", "attend_rows(c, qrow, K, V, b, g / G, ctx_len", "attend_rows(c, qrow, K, V, b, g % c->Hkv, ctx_len"),
    ("GQA map of logits", "      const int h = g / G;\n      const uint16_t* qrow = q + ((int64_t)b * c->Hq + g) * c->d;\n      double* out = logits",
     "      const int h = g % c->Hkv;\n      const uint16_t* qrow = q + ((int64_t)b * c->Hq + g) * c->d;\n      double* out = logits"),
    ("recent window start", "for (int64_t j = recent_start[b] < 0 ? 0 : recent_start[b]; j < L; ++j) take[j] = 1;",
     "for (int64_t j = recent_start[b] + 1; j < L; ++j) take[j] = 1;"),
    ("sink rows", "for (int64_t j = 0; j < c->n_sink && j < L; ++j) take[j] = 1;",
     "for (int64_t j = 0; j + 1 < c->n_sink && j < L; ++j) take[j] = 1;"),
    ("V addressed with K's strides", "return V + b * c->v_stride_b + h * c->v_stride_h + j * c->v_stride_t;",
     "return V + b * c->k_stride_b + h * c->k_stride_h + j * c->k_stride_t;"),
    # attention arithmetic
    ("logit scale dropped", "return c->scale * s;", "return s;"),
    ("output not normalised", "    for (int t = 0; t < c->d; ++t) out[t] /= Z;", "    for (int t = 0; t < c->d; ++t) out[t] /= 1.0;"),
    # evidence
    ("softmax over the prefix instead of J", "for (int64_t j = j_lo; j < j_end; ++j) Z += exp(l[j] - M);",
     "for (int64_t j = 0; j < L; ++j) Z += exp(l[j] - M);"),
    # (dropping the 1 / G of Eq. selector_mu is not a mistake anything downstream can see: Eq. selector_f
    # normalises, so a constant factor of mu cancels -- not listed)
    ("power of the evidence dropped", "mu[j - j_lo] += pow(p, c->alpha) / (double)G;", "mu[j - j_lo] += p / (double)G;"),
    ("inverse power map", "f[i] = pow(mu[i], 1.0 / c->alpha);", "f[i] = pow(mu[i], c->alpha);"),
    ("causal mask ignored", "if (vis && vis[(int64_t)b * c->Hq + h * G + gg] < j_end) j_end", "if (0 && vis[(int64_t)b * c->Hq + h * G + gg] < j_end) j_end"),
    ("causal mask off by one", "j_end = vis[(int64_t)b * c->Hq + h * G + gg];", "j_end = vis[(int64_t)b * c->Hq + h * G + gg] + 1;"),
    # prior
    ("key-norm exponent sign", "pow(kn + eps, -c->gamma)", "pow(kn + eps, c->gamma)"),
    ("epsilon of the key-norm factor", "pow(kn + eps, -c->gamma)", "pow(kn, -c->gamma)"),
    ("epsilon of u", "/ (jmax - jmin + eps);", "/ (jmax - jmin);"),
    ("decay exponent p", "exp(-c->beta * pow(u, c->p))", "exp(-c->beta * u)"),
    ("decay sign", "exp(-c->beta * pow(u, c->p))", "exp(c->beta * pow(u, c->p))"),
    ("epsilon of the tail brake", "pow(1.0 - u + eps, c->eta)", "pow(1.0 - u, c->eta)"),
    ("prior not normalised", "for (int64_t i = 0; i < nJ; ++i) r[i] /= rs;", "for (int64_t i = 0; i < nJ; ++i) r[i] /= 1.0;"),
    # fusion
    ("lambda* denominator", "lambda = den > 1e-300 ? (ff - fr) / den : 0.0;", "lambda = den > 1e-300 ? (ff - fr) / (ff + rr) : 0.0;"),
    ("lambda* zero-denominator guard", "lambda = den > 1e-300 ? (ff - fr) / den : 0.0;", "lambda = (ff - fr) / den;"),
    ("lambda* lower clip", "if (lambda < 0.0) lambda = 0.0;", ""),
    ("lambda* upper clip", "if (lambda > c->lambda_clip) lambda = c->lambda_clip;", ""),
    ("mixture weights swapped", "sc[i] = (1.0 - lambda) * f[i] + lambda * r[i];", "sc[i] = lambda * f[i] + (1.0 - lambda) * r[i];"),
    ("epsilon of the log score", "z[(int64_t)h * nJ + i] = log(sc[i] + eps);", "z[(int64_t)h * nJ + i] = log(sc[i]);"),
    # refinements
    ("Soft-NMS sign", "zn[i] = zh[i] - c->alpha_soft * (gap > 0.0 ? gap : 0.0);", "zn[i] = zh[i] + c->alpha_soft * (gap > 0.0 ? gap : 0.0);"),
    ("Soft-NMS window one short", "t <= i + c->nms_radius; ++t)", "t < i + c->nms_radius; ++t)"),
    ("head-softmax temperature", "zc[h] = z[(int64_t)h * nJ + i] / c->temp;", "zc[h] = z[(int64_t)h * nJ + i] * c->temp;"),
    ("responsibility floor", "if (resp < eps) resp = eps;", ""),
    ("cross-head sign", "z[(int64_t)h * nJ + i] += c->alpha_cross * log(resp);", "z[(int64_t)h * nJ + i] -= c->alpha_cross * log(resp);"),
    # Top-K
    ("tie-break", "return (x->j > y->j) - (x->j < y->j);", "return (x->j < y->j) - (x->j > y->j);"),
    ("ranking order", "  if (x->z > y->z) return -1;\n  if (x->z < y->z) return 1;", "  if (x->z > y->z) return 1;\n  if (x->z < y->z) return -1;"),
    ("output not ascending", "qsort(s, (size_t)k_take, sizeof(int32_t), cmp_i32);", ""),
    # key norms, Reorg, trigger, state update, decode loop
    ("key norm without the root", "knorm[((int64_t)b * c->Hkv + h) * ld + j] = sqrt(s);", "knorm[((int64_t)b * c->Hkv + h) * ld + j] = s;"),
    ("Reorg target row", "memcpy(kc + (c->n_sink + i) * c->d, k_row(c, K, b, h, j)", "memcpy(kc + i * c->d, k_row(c, K, b, h, j)"),
    ("trigger looks at the current token", "if (trig[i] == x[t - 1]) slow = 1;", "if (trig[i] == x[t]) slow = 1;"),
    ("forced refresh one step late", "if (fast_run >= t_max) slow = 1;", "if (fast_run > t_max) slow = 1;"),
    ("first step not slow", "    if (t == 0) {\n      slow = 1;", "    if (t == 0) {\n      slow = 0;"),
    ("window does not respect the sink", "recent_start[b] = L - c->recent > c->n_sink ? L - c->recent : c->n_sink;", "recent_start[b] = L - c->recent;"),
    ("window slides before the row is counted", "recent_start[b] = L - c->recent > c->n_sink ? L - c->recent : c->n_sink;",
     "recent_start[b] = L - 1 - c->recent > c->n_sink ? L - 1 - c->recent : c->n_sink;"),
    ("fast step refreshes the set", "      if (g[(int64_t)t * c->B + b]) {\n        rc |= sfio_dense(&c1, qb, Kb, Vb, ctx_len + b, ob);",
     "      if (1) {\n        rc |= sfio_dense(&c1, qb, Kb, Vb, ctx_len + b, ob);"),
]


def _build(src_text, path_c, path_so):
    with open(path_c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", path_c, "-o", path_so, "-lm"],
                   check=True, capture_output=True)


def _pins_pass(path_so):
    env = dict(os.environ, SFI_ORACLE_LIB=path_so, OMP_NUM_THREADS="1")
    try:
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES], cwd=HERE, env=env,
                           capture_output=True, text=True, timeout=300)
    except subprocess.TimeoutExpired:  # a planted mistake that never ends is a noticed one
        return False, "timeout"
    return r.returncode == 0, r.stdout[-400:]


def test_every_planted_mistake_is_noticed(tmp_path):
    if os.environ.get("SFI_ORACLE_LIB"):
        pytest.skip("already running against a planted mistake")
    src = open(SRC).read()
    jobs = [("unchanged", src)]
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, f"mutant '{name}': its text occurs {src.count(old)} times in sfi_oracle.c"
        jobs.append((name, src.replace(old, new)))

    def run(i):
        name, text = jobs[i]
        so = str(tmp_path / f"m{i}.so")
        _build(text, str(tmp_path / f"m{i}.c"), so)
        return name, _pins_pass(so)

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        results = list(ex.map(run, range(len(jobs))))
    name, (ok, tail) = results[0]
    assert ok, f"the unchanged oracle fails its pins when built here:\n{tail}"
    survivors = [name for name, (ok, _) in results[1:] if ok]
    assert not survivors, f"planted mistakes no pin noticed: {survivors}"
