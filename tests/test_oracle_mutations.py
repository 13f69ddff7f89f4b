"""The pins must bite: plant one plausible mistake at a time in a copy of the oracle's C source,
build it, and check that the pin suite (tests/test_oracle_pins.py) fails against it.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mmse_oracle.c")

MUTATIONS = [
    ("residual sign flipped", "float r = fmaf(-alpha, q, x[i]);", "float r = fmaf(alpha, q, x[i]);"),
    ("square term dropped", "s = fmaf(r, r, s);", "s = s + r;"),
    ("upper saturation dropped", "    if (q > hi) q = hi;\n    return q;\n}\n\n/* Integer code", "    return q;\n}\n\n/* Integer code"),
    ("lower saturation dropped in the definition", "    if (q < (double)qmin) q = (double)qmin;", "    ;"),
    ("round half away from zero", "return can_clamp(rintf(x * inv), lo, hi);", "return can_clamp(roundf(x * inv), lo, hi);"),
    ("grid misses the max-abs scale", "float frac = (float)(j + 1) / (float)G;", "float frac = (float)(j) / (float)G + 0.001f;"),
    ("abs-max without the absolute value", "float v = fabsf(x[i]);", "float v = x[i];"),
    ("argmin keeps the last of equal minima", "if (e[j] < e[jb]) jb = j;", "if (e[j] <= e[jb]) jb = j;"),
    ("argmax instead of argmin", "if (e[j] < e[jb]) jb = j;", "if (e[j] > e[jb]) jb = j;"),
    ("pairwise sum drops the unpaired value", "if (m & 1) v[h] = v[m - 1];", "if (m & 1) v[h] = 0.0;"),
    ("last partial chunk skipped", "const int64_t m = (n + ORACLE_CHUNK - 1) / ORACLE_CHUNK;\n#pragma omp parallel for schedule(static) if (m > 4096)",
     "const int64_t m = (n + ORACLE_CHUNK - 1) / ORACLE_CHUNK;\n    if (n % ORACLE_CHUNK) { work[m - 1] = 0.0; }\n#pragma omp parallel for schedule(static) if (m > 4096)\n    for (int64_t c = 0; c < n / ORACLE_CHUNK; ++c) {\n        work[c] = (double)can_chunk_sse(x + c * ORACLE_CHUNK, ORACLE_CHUNK, alpha, inv, lo, hi);\n    }\n    if (0)"),
    ("refinement bracket one grid step too low", "float hi = (j == G - 1) ? a_j : can_grid_alpha(absmax, qmax, G, j + 1);",
     "float hi = a_j;"),
    ("refinement forgets the grid point", "float best_a = a_j;\n    double best = e_j;", "float best_a = a_j;\n    double best = 1e300;"),
    ("refinement keeps the wrong half", "if (ec <= ed) {\n                hi = d;", "if (ec > ed) {\n                hi = d;"),
    ("nibbles swapped", "packed[b] = (uint8_t)(lo | (hi << 4));", "packed[b] = (uint8_t)(hi | (lo << 4));"),
    ("unpack without sign extension", "if (is_signed && v >= 8) v -= 16;", ";"),
    ("rows of a tensor read transposed", "can_search(w + k * n, n,", "can_search(w + (K - 1 - k) * n, n,"),
    ("one scale for every row when coding", "float inv = 1.0f / scale[k];\n        for (int64_t i = 0; i < n; ++i)\n            codes[k * n + i]",
     "float inv = 1.0f / scale[0];\n        for (int64_t i = 0; i < n; ++i)\n            codes[k * n + i]"),
    ("residual uses the wrong sign", "resid[k * n + i] = fmaf(-a1, can_code(x, inv, lo, hi), x);", "resid[k * n + i] = fmaf(a1, can_code(x, inv, lo, hi), x);"),
    ("second tensor searched on the weights, not the residual", "can_search_kernelwise(resid, K, n, qmin, qmax, G, iters, scale2, idx2, sse2);",
     "can_search_kernelwise(w, K, n, qmin, qmax, G, iters, scale2, idx2, sse2);"),
    ("alternating: first half-step fits the residual of the wrong tensor",
     "        can_subtract_codes(t, q2, a2, n, r);\n        if (can_phi(r, n, qmin, qmax, G, iters, &ta1, tq1, &te1) != 0) break;",
     "        can_subtract_codes(t, q1, a1, n, r);\n        if (can_phi(r, n, qmin, qmax, G, iters, &ta1, tq1, &te1) != 0) break;"),
    ("alternating: second half-step fits the weights, not the residual",
     "        can_subtract_codes(t, tq1, ta1, n, r);", "        can_subtract_codes(t, tq1, 0.0f, n, r);"),
    ("alternating: residual added instead of subtracted",
     "out[i] = fmaf(-alpha, (float)q[i], t[i]);", "out[i] = fmaf(alpha, (float)q[i], t[i]);"),
    ("alternating: worse sweeps are kept", "if (!(te < e)) break;", ";"),
    ("alternating: stopping rule ignored", "if (conv) break;", ";"),
    ("dual search: only the rounded first code is tried", "    for (int t = qmin; t <= qmax; ++t) {\n        float r = fmaf(-a1, (float)t, x);",
     "    for (int t = (int)can_clamp(rintf(x / a1), lo, hi); t <= (int)can_clamp(rintf(x / a1), lo, hi); ++t) {\n        float r = fmaf(-a1, (float)t, x);"),
    ("dual search: second code not saturated in the definition", "double d = r - a2 * def_round_sat(r / a2, qmin, qmax);", "double d = r - a2 * nearbyint(r / a2);"),
    ("dual search: second scale grid is absolute, not relative", "return a1 * frac;", "return frac;"),
    ("dual search: last of equal minima", "if (e < best) { best = e; ba = ja; bb = jb; }", "if (e <= best) { best = e; ba = ja; bb = jb; }"),
    ("dual search: codes of the wrong scale pair", "can_dual_codes(x, n, *a1_out, *a2_out, qmin, qmax, q1, q2);", "can_dual_codes(x, n, *a1_out, *a1_out, qmin, qmax, q1, q2);"),
    ("dual search: highest code wins ties", "if (e < best) { best = e; bt = t; bq = (int)q; }", "if (e <= best) { best = e; bt = t; bq = (int)q; }"),
    ("activation residual: second tensor saturated to the first range",
     "int rc = can_search(resid, N, qmin2, qmax2, G, iters, beta2, idx2, sse2, NULL, NULL);",
     "int rc = can_search(resid, N, qmin1, qmax1, G, iters, beta2, idx2, sse2, NULL, NULL);"),
    ("activation residual: first tensor saturated to the second range",
     "can_residual(x, 1, N, &beta1, qmin1, qmax1, resid);", "can_residual(x, 1, N, &beta1, qmin2, qmax2, resid);"),
    ("activation residual: codes of the input, not of the residual",
     "if (packed2) can_quantize_pack_int4(resid, 1, N, beta2, qmin2, qmax2, packed2);",
     "if (packed2) can_quantize_pack_int4(x, 1, N, beta2, qmin2, qmax2, packed2);"),
    ("offset: delta is the maximum", "if (x[i] < m) m = x[i];\n    }\n    return bad ? NAN : m;", "if (-x[i] < m) m = -x[i];\n    }\n    return bad ? NAN : -m;"),
    ("offset: delta added, not subtracted", "for (int64_t i = 0; i < N; ++i) y[i] = x[i] - d;", "for (int64_t i = 0; i < N; ++i) y[i] = x[i] + d;"),
    ("offset: shifted tensor searched in a signed range", "int rc = can_search(y, N, 0, qmax, G, iters, scale, idx, sse, NULL, NULL);",
     "int rc = can_search(y, N, -qmax / 2 - 1, qmax / 2, G, iters, scale, idx, sse, NULL, NULL);"),
    ("offset: definition forgets to add delta back", "double that = alpha * def_round_sat(((double)x[i] - delta) / alpha, 0, qmax) + delta;",
     "double that = alpha * def_round_sat(((double)x[i] - delta) / alpha, 0, qmax);"),
    ("offset: codes of the unshifted tensor", "if (packed) can_quantize_pack_int4(y, 1, N, scale, 0, qmax, packed);",
     "if (packed) can_quantize_pack_int4(x, 1, N, scale, 0, qmax, packed);"),
    ("offset: non-finite input accepted", "*delta = rc == 0 ? d : NAN;", "*delta = d;"),
    ("comparison: alternating update divides by the sum of |codes|", "den += (int64_t)q * (int64_t)q;", "den += (int64_t)fabsf(q);"),
    ("comparison: alternating numerator uses the codes twice", "num = fma((double)x[s0 + i], (double)q, num);",
     "num = fma((double)q, (double)q, num);"),
    ("comparison: alternating update inverted", "float next = (float)(num / (double)den);", "float next = (float)((double)den / num);"),
    ("comparison: alternating starts from half the max-abs scale", "float alpha = a / (float)qmax;\n        for (int it = 0; it < max_iters; ++it) {",
     "float alpha = 0.5f * a / (float)qmax;\n        for (int it = 0; it < max_iters; ++it) {"),
    ("comparison: alternating stops after one update", "alpha = next;\n            *updates = it + 1;", "alpha = next;\n            *updates = it + 1; break;"),
    ("comparison: alternating keeps the old scale", "alpha = next;\n            *updates = it + 1;", "*updates = it + 1;"),
    ("tiny tensors not special-cased", "} else if (a < ORACLE_TINY) {\n        *scale = 1.0f; *idx = 0;",
     "} else if (a < 0.0f) {\n        *scale = 1.0f; *idx = 0;"),
    ("dual search: tiny tensors not special-cased", "} else if (a < ORACLE_TINY) {\n        *a1_out = 1.0f;",
     "} else if (a < 0.0f) {\n        *a1_out = 1.0f;"),
    ("non-finite input accepted", "return bad ? NAN : a;", "return a;"),
]


@pytest.fixture(scope="module")
def source():
    return open(SRC).read()


def test_unmutated_oracle_passes_its_pins(tmp_path):
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_mutation(tmp_path, source, name, old, new):
    from oracle import build as oracle_build
    assert source.count(old) == 1, f"mutation anchor not unique for: {name}"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(source.replace(old, new))
    lib = str(tmp_path / "libmutant.so")
    oracle_build.build(src=str(mutated), out=lib)
    env = dict(os.environ, MMSE_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env,
                       capture_output=True, text=True)
    assert r.returncode != 0, f"no pin noticed: {name}"
