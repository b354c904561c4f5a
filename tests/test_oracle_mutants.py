"""Mutation check of the oracle's pins: every planted mistake must fail a pin.

For each entry of MUTANTS the test writes a copy of ``oracle/pulsed_update_oracle.c`` with one
expression changed (a swapped operand, a wrong index, a dropped term, a flipped sign ...), builds
it in a temporary directory and runs the oracle's own pins (``tests/test_oracle_*.py``, CPU only)
against that build in a child process.  The pins must fail; a mutant that passes them names a
part of the oracle that nothing but itself defines.  The unchanged source must pass.  The
Python-level compositions of ``oracle/__init__.py`` (unit cells) are mutated in-process.

The original snippets are looked up literally: a change to the oracle that removes one makes
this test fail until the list follows.
"""
import concurrent.futures
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pulsed_update_oracle.c")
GCC = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]

# (function, planted mistake, original, mutated)
MUTANTS = [
    ("orc_philox4x32_10", "second key word dropped from the round",
     "uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;", "uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k0;"),
    ("orc_philox4x32_10", "nine rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
    ("orc_philox4x32_10", "multipliers swapped",
     "const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;", "const uint64_t M1 = 0xD2511F53u, M0 = 0xCD9E8D57u;"),
    ("orc_gauss_block_f64", "step missing from the counter",
     "ctr[0] = index; ctr[1] = blk; ctr[2] = t; ctr[3] = tag << 24;", "ctr[0] = index; ctr[1] = blk; ctr[2] = 0; ctr[3] = tag << 24;"),
    ("orc_gauss_block_f64", "sine where the cosine belongs",
     "z[2 * pair] = rad * cos(two_pi * u2);", "z[2 * pair] = rad * sin(two_pi * u2);"),
    ("orc_gauss_block_f64", "both uniforms from one word",
     "double u1 = ((double)(r[2 * pair] >> 8) + 1.0) / 16777216.0;", "double u1 = ((double)(r[2 * pair + 1] >> 8) + 1.0) / 16777216.0;"),
    ("orc_gauss_block_f64", "u1 may reach zero",
     "double u1 = ((double)(r[2 * pair] >> 8) + 1.0) / 16777216.0;", "double u1 = ((double)(r[2 * pair] >> 8) + 0.0) / 16777216.0;"),
    ("orc_gauss", "wrong number of the block", "return (float)z[q & 3];", "return (float)z[(q + 1) & 3];"),
    ("orc_device_planes", "step may turn negative",
     "float dw = dw_min * fabsf(1.0f + dw_min_dtod * g[0]);", "float dw = dw_min * (1.0f + dw_min_dtod * g[0]);"),
    ("orc_device_planes", "asymmetry with one sign", "dw_down[k] = dw * (1.0f - a);", "dw_down[k] = dw * (1.0f + a);"),
    ("orc_device_planes", "slope of the lower bound with the wrong sign",
     "sd = (bmin != 0.0f) ? gd / bmin : 0.0f;", "sd = (bmin != 0.0f) ? gd / -bmin : 0.0f;"),
    ("orc_device_planes", "both bounds from one Gaussian",
     "float bmin = fminf(0.0f, w_min * (1.0f + w_min_dtod * g[3]));", "float bmin = fminf(0.0f, w_min * (1.0f + w_min_dtod * g[2]));"),
    ("orc_line_scale_ex", "update management inverted", "a_x[b] = A * sqrt(m_d / m_x);", "a_x[b] = A * sqrt(m_x / m_d);"),
    ("orc_line_scale_ex", "train length missing from the probability factor",
     "double A = sqrt((double)lr / ((double)dw_min * (double)bl));", "double A = sqrt((double)lr / ((double)dw_min));"),
    ("orc_line_scale_ex", "variable length rounded down",
     "double need = ceil((double)lr * m_x * m_d / (double)dw_min);", "double need = floor((double)lr * m_x * m_d / (double)dw_min);"),
    ("orc_line_scale_ex", "non-finite entries enter the maxima",
     "static int is_active(float v) { return isfinite(v) && v != 0.0f; }", "static int is_active(float v) { return v != 0.0f; }"),
    ("orc_threshold", "saturation just below one", "if (!(p < 1.0)) p = 1.0; ", "if (!(p < 1.0)) p = 0.99999999; "),
    ("orc_threshold", "31-bit threshold", "return (uint64_t)floor(p * 4294967296.0);", "return (uint64_t)floor(p * 2147483648.0);"),
    ("orc_pulse_word", "line and sample swapped in the counter",
     "ctr[0] = index; ctr[1] = b; ctr[2] = t; ctr[3] = (tag << 24) | (uint32_t)(n >> 2);",
     "ctr[0] = b; ctr[1] = index; ctr[2] = t; ctr[3] = (tag << 24) | (uint32_t)(n >> 2);"),
    ("orc_pulse_word", "<= in place of <", "if ((uint64_t)r[n & 3] < T)", "if ((uint64_t)r[n & 3] <= T)"),
    ("orc_pulse_word", "wrong word of the block", "if ((uint64_t)r[n & 3] < T)", "if ((uint64_t)r[(n + 1) & 3] < T)"),
    ("orc_pulse_word", "sign bit inverted",
     "    if (v < 0.0f) word |= (uint64_t)1 << 63;\n    return word;\n}\n\n/* Deterministic",
     "    if (v > 0.0f) word |= (uint64_t)1 << 63;\n    return word;\n}\n\n/* Deterministic"),
    ("bit_reverse32", "31 of 32 bits reversed", "for (int k = 0; k < 32; ++k) { r = (r << 1) | (v & 1u); v >>= 1; }",
     "for (int k = 0; k < 31; ++k) { r = (r << 1) | (v & 1u); v >>= 1; }"),
    ("orc_pulse_word_deterministic", "no digital shift on the row trains",
     "else set = (uint64_t)(bit_reverse32((uint32_t)n) ^ 0xAAAAAAAAu) < T;", "else set = (uint64_t)(bit_reverse32((uint32_t)n)) < T;"),
    ("orc_pulse_word_deterministic", "column pulses at the start of their slots",
     "set = (((uint64_t)(2 * n + 1)) << 32) < 2u * (uint64_t)BL * T;", "set = (((uint64_t)(2 * n)) << 32) < 2u * (uint64_t)BL * T;"),
    ("orc_pulse_words_ex", "row trains drawn with the column tag",
     ": orc_pulse_word(seed, t, ORC_TAG_D, (uint32_t)i, (uint32_t)b, a_d[b], v, bl_b[b]);",
     ": orc_pulse_word(seed, t, ORC_TAG_X, (uint32_t)i, (uint32_t)b, a_d[b], v, bl_b[b]);"),
    ("orc_pulse_words_ex", "row trains scaled with the column factor",
     ": orc_pulse_word(seed, t, ORC_TAG_D, (uint32_t)i, (uint32_t)b, a_d[b], v, bl_b[b]);",
     ": orc_pulse_word(seed, t, ORC_TAG_D, (uint32_t)i, (uint32_t)b, a_x[b], v, bl_b[b]);"),
    ("coincidences", "direction inverted",
     "*up = (int)(((xword ^ dword) >> 63) & 1);", "*up = 1 - (int)(((xword ^ dword) >> 63) & 1);"),
    ("coincidences", "sign bits counted as a pulse", "uint64_t both = xword & dword & mask;", "uint64_t both = xword & dword;"),
    ("orc_counts", "sign of the count inverted", "signed_counts[(size_t)i * C + j] = (int8_t)(up ? n : -n);",
     "signed_counts[(size_t)i * C + j] = (int8_t)(up ? -n : n);"),
    ("orc_counts", "rows and columns transposed",
     "int n = coincidences(xw[(size_t)b * C + j], dw[(size_t)b * R + i], BL, &up);\n            signed_counts",
     "int n = coincidences(xw[(size_t)b * C + i], dw[(size_t)b * R + j], BL, &up);\n            signed_counts"),
    ("orc_device_step", "up and down step sizes swapped", "float s = up ? s_up : s_dn;", "float s = up ? s_dn : s_up;"),
    ("orc_device_step", "up and down slopes swapped", "float slope = up ? slope_up : slope_dn;", "float slope = up ? slope_dn : slope_up;"),
    ("orc_device_step", "noise with the wrong sign", "float noise = 1.0f + cx;", "float noise = 1.0f - cx;"),
    ("orc_device_step", "lower clip at minus the upper bound", "wn = fmaxf(wn, bmin);", "wn = fmaxf(wn, -bmax);"),
    ("orc_device_step", "step may reverse through the slope", "f = fmaxf(0.0f, 1.0f - prod);", "f = 1.0f - prod;"),
    ("orc_apply_words", "noise indexed by block number, not pulse number",
     "if ((q & 3) == 0) orc_gauss_block_f64(seed, cell, t, q >> 2, ORC_TAG_C2C, zblk);",
     "if ((q & 3) == 0) orc_gauss_block_f64(seed, cell, t, q, ORC_TAG_C2C, zblk);"),
    ("orc_apply_words", "samples applied in reverse order",
     "xwT[(size_t)j * B + b] = xw[(size_t)b * C + j];", "xwT[(size_t)j * B + b] = xw[(size_t)(B - 1 - b) * C + j];"),
    ("orc_apply_words", "pulse counter restarts with every sample",
     "        for (int b = 0; b < B; ++b) {\n            int up;", "        for (int b = 0; b < B; ++b) {\n            q = 0;\n            int up;"),
    ("orc_pulsed_update_ex", "words of the step before",
     "orc_pulse_words_ex(x, d, B, R, C, lr, dw_min, BL, update_management, train_kind, dynamic_bl, seed,\n                       t, xw, dw);",
     "orc_pulse_words_ex(x, d, B, R, C, lr, dw_min, BL, update_management, train_kind, dynamic_bl, seed,\n                       t + 1u, xw, dw);"),
    ("orc_temporal_planes", "decay and diffusion planes from one Gaussian",
     "float g8 = orc_gauss(seed, cell, 0u, 7u, ORC_TAG_D2D);", "float g8 = orc_gauss(seed, cell, 0u, 6u, ORC_TAG_D2D);"),
    ("orc_temporal_planes", "decay rate not clipped", "lam = fminf(fmaxf(lam, 0.0f), 1.0f);", "lam = fmaxf(lam, 0.0f);"),
    ("temporal_gauss", "temporal step missing from the stream",
     "return orc_gauss(seed, 0u, tau, cell, tag);", "return orc_gauss(seed, 0u, 0u, cell, tag);"),
    ("orc_decay_diffuse", "decay toward the wrong side", "float keep = 1.0f - lambda[k];", "float keep = 1.0f + lambda[k];"),
    ("orc_decay_diffuse", "no upper clip after diffusion",
     "        w = w + dz;\n        w = fmaxf(w, b_min[k]);\n        w = fminf(w, b_max[k]);", "        w = w + dz;\n        w = fmaxf(w, b_min[k]);"),
    ("orc_reset_columns", "reset noise from the diffusion stream",
     "float xi = temporal_gauss(seed, (uint32_t)k, tau, ORC_TAG_RESET);", "float xi = temporal_gauss(seed, (uint32_t)k, tau, ORC_TAG_DIFFUSION);"),
    ("orc_reset_columns", "one column too many", "for (int j = c0; j < c0 + ncols && j < C; ++j) {", "for (int j = c0; j <= c0 + ncols && j < C; ++j) {"),
    ("analog_mvm", "transposed product reads the matrix untransposed",
     "size_t cell = transposed ? (size_t)j * C + i : (size_t)i * C + j;", "size_t cell = transposed ? (size_t)i * C + j : (size_t)i * C + j;"),
    ("analog_mvm", "rounding toward zero in the DAC", "if (inp_res > 0.0f) xh = rintf(xh / inp_res) * inp_res;", "if (inp_res > 0.0f) xh = truncf(xh / inp_res) * inp_res;"),
    ("analog_mvm", "output noise keyed without the vector",
     "orc_gauss_block_f64(seed, (uint32_t)i >> 1, t, (uint32_t)b, tag_out, zb);", "orc_gauss_block_f64(seed, (uint32_t)i >> 1, t, 0u, tag_out, zb);"),
    ("analog_mvm", "weight noise not scaled by the input norm", "float wn = w_noise * norm;", "float wn = w_noise;"),
    ("analog_mvm", "weight and output noise from one Gaussian",
     "float g_out = (float)zb[2 * (i & 1)], g_w = (float)zb[2 * (i & 1) + 1];", "float g_out = (float)zb[2 * (i & 1)], g_w = (float)zb[2 * (i & 1)];"),
    ("analog_mvm", "no clipping in the ADC", "float q = fminf(fmaxf(z, -out_bound), out_bound);", "float q = z;"),
    ("analog_mvm", "dynamic scale not returned to the output", "y[(size_t)b * N + i] = alpha * q;", "y[(size_t)b * N + i] = q;"),
    ("analog_mvm", "input noise added before the DAC rounds it away",
     "            xq[j] = xh;\n        }\n        if (inp_noise > 0.0f) {", "            xq[j] = xh;\n        }\n        if (inp_noise > 0.0f && inp_res == 0.0f) {"),
    ("analog_mvm", "cellwise weight noise shared by the vectors of a batch",
     "orc_gauss_block_f64(seed, (uint32_t)cell, t, (uint32_t)b, transposed ? 12u : 11u, zc);",
     "orc_gauss_block_f64(seed, (uint32_t)cell, t, 0u, transposed ? 12u : 11u, zc);"),
    ("orc_conv_patches", "kernel row and column swapped",
     "int iy = oy * stride - pad + ky, ix = ox * stride - pad + kx;", "int iy = oy * stride - pad + kx, ix = ox * stride - pad + ky;"),
    ("orc_conv_patches", "padding ignored", "int iy = oy * stride - pad + ky, ix = ox * stride - pad + kx;", "int iy = oy * stride + ky, ix = ox * stride + kx;"),
    ("orc_conv_rows", "output positions transposed",
     "d[b * Cout + i] = dgrad[(((size_t)n * Cout + i) * OH + oy) * OW + ox];", "d[b * Cout + i] = dgrad[(((size_t)n * Cout + i) * OH + ox) * OW + oy];"),
]

# Python-level compositions: (function, planted mistake, original, mutated, pins that must fail)
PY_MUTANTS = [
    ("unit_cell_update", "every device draws its own pulse trains",
     "xw, dw = pulse_words(x, d, lr, params[0].dw_min, BL, update_management, seeds[0], t)\n    counts = []\n    for k, W in enumerate(Ws):",
     "counts = []\n    for k, W in enumerate(Ws):\n        xw, dw = pulse_words(x, d, lr, params[k].dw_min, BL, update_management, seeds[k], t)"),
    ("unit_cell_update", "one-by-one update ignores the choice", "if which >= 0 and k != which:", "if which >= 0 and k != which and False:"),
    ("unit_cell_update", "all devices share the first one's noise stream",
     "xw, dw, BL, seeds[k], t))", "xw, dw, BL, seeds[0], t))"),
    ("unit_cell_weights", "factors ignored", "acc = (acc + np.float32(g) * W.astype(np.float32)).astype(np.float32)",
     "acc = (acc + W.astype(np.float32)).astype(np.float32)"),
]


# where a function's pins mostly live: that file runs first, the others only if it passes
PINS_OF = {"orc_philox4x32_10": "test_oracle_philox.py", "orc_gauss_block_f64": "test_oracle_philox.py",
           "orc_gauss": "test_oracle_philox.py", "orc_device_planes": "test_oracle_device.py",
           "orc_device_step": "test_oracle_device.py", "orc_apply_words": "test_oracle_device.py",
           "orc_line_scale_ex": "test_oracle_train_modes.py", "bit_reverse32": "test_oracle_train_modes.py",
           "orc_pulse_word_deterministic": "test_oracle_train_modes.py", "orc_temporal_planes": "test_oracle_temporal.py",
           "temporal_gauss": "test_oracle_temporal.py", "orc_decay_diffuse": "test_oracle_temporal.py",
           "orc_reset_columns": "test_oracle_temporal.py", "analog_mvm": "test_oracle_mvm.py",
           "orc_conv_patches": "test_oracle_conv.py", "orc_conv_rows": "test_oracle_conv.py"}


def _run_pins(lib_path, first=None):
    env = dict(os.environ, AHT_ORACLE_LIB=lib_path, OMP_NUM_THREADS="2")
    base = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"]
    runs = []
    if first:
        runs.append(base + [os.path.join(ROOT, "tests", first)])
    runs.append(base + [os.path.join(ROOT, "tests"), "-k", "oracle and not mutants and not sanitizer"])
    for cmd in runs:
        r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            break
    failed = [l for l in r.stdout.splitlines() if l.startswith("FAILED")]
    return r.returncode, (failed[0] if failed else r.stdout[-400:])


def _build(src_text, tmp, tag):
    c = os.path.join(tmp, f"oracle_{tag}.c")
    so = os.path.join(tmp, f"liboracle_{tag}.so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(GCC + ["-o", so, c, "-lm"], check=True)
    return so


def test_every_planted_mistake_in_the_c_oracle_fails_a_pin(tmp_path):
    orig = open(SRC).read()
    for fn, what, a, b in MUTANTS:
        assert orig.count(a) >= 1, f"{fn}: snippet not found (the oracle changed; update the list): {a!r}"
    rc, msg = _run_pins(_build(orig, str(tmp_path), "control"))
    assert rc == 0, f"the unchanged oracle fails its pins: {msg}"

    def one(k):
        fn, what, a, b = MUTANTS[k]
        so = _build(orig.replace(a, b, 1), str(tmp_path), f"m{k}")
        return k, _run_pins(so, PINS_OF.get(fn, "test_oracle_trains.py"))

    survivors, broken = [], []
    with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, min(6, (os.cpu_count() or 2) - 1))) as pool:
        for k, (rc, msg) in pool.map(one, range(len(MUTANTS))):
            fn, what = MUTANTS[k][0], MUTANTS[k][1]
            if rc == 0:
                survivors.append(f"{fn}: {what}")
            elif rc != 1:                                  # not a test failure: collection error, crash ...
                broken.append(f"{fn}: {what}: rc {rc}: {msg}")
    assert not broken, broken
    assert not survivors, f"planted mistakes that no pin notices: {survivors}"
    functions = {m[0] for m in MUTANTS}
    print(f"{len(MUTANTS)} mutants in {len(functions)} functions, none alive")


@pytest.mark.parametrize("k", range(len(PY_MUTANTS)), ids=[f"{m[0]}-{i}" for i, m in enumerate(PY_MUTANTS)])
def test_every_planted_mistake_in_the_unit_cell_composition_fails_a_pin(k, monkeypatch):
    import oracle
    import test_oracle_unit_cell as pins
    fn, what, a, b = PY_MUTANTS[k]
    path = os.path.join(ROOT, "oracle", "__init__.py")
    text = open(path).read()
    assert text.count(a) == 1, f"{fn}: snippet not found (the oracle changed; update the list)"
    spec = importlib.util.spec_from_loader("oracle_mutant", loader=None)
    mod = importlib.util.module_from_spec(spec)
    mod.__file__ = path
    monkeypatch.setitem(sys.modules, "oracle_mutant", mod)     # dataclasses look their module up
    exec(compile(text.replace(a, b), path, "exec"), mod.__dict__)
    monkeypatch.setattr(oracle, fn, getattr(mod, fn))
    failed = 0
    for name in dir(pins):
        if name.startswith("test_"):
            try:
                getattr(pins, name)()
            except AssertionError:
                failed += 1
    assert failed > 0, f"{fn}: {what}: no pin notices"
