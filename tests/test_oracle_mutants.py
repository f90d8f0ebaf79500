"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the
oracle's C source (a wrong ring direction, a dropped truncation, a different
tie rule, a sign error, ...), builds it, and runs the pin tests against that
build in a subprocess: at least one pin must fail.  The planted mistakes live
only in temporary copies; the committed oracle is never modified.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pipesgd_oracle.c")

PIN_FILES = ["tests/test_oracle_codec.py", "tests/test_oracle_ring.py", "tests/test_oracle_update.py",
             "tests/test_oracle_bucket.py", "tests/test_oracle_direct.py", "tests/test_oracle_hd.py", "tests/test_golden.py"]

# (name, text to find, replacement)
MUTANTS = [
    ("receive_from_the_wrong_neighbour",
     "const orc_msg *m = &R->wire[modp(r - 1, p)];", "const orc_msg *m = &R->wire[modp(r + 1, p)];"),
    ("send_the_wrong_block",
     "for (int r = 0; r < p; ++r) ring_send(R, r, modp(r - s, p));",
     "for (int r = 0; r < p; ++r) ring_send(R, r, modp(r + s, p));"),
    ("owner_off_by_one",
     "int orc_ring_owner_chunk(const orc_ring *R, int r) { return modp(r + 1, R->p); }",
     "int orc_ring_owner_chunk(const orc_ring *R, int r) { return modp(r, R->p); }"),
    ("truncation_rounds_to_nearest",
     "static uint16_t trunc16_c(float x) { return (uint16_t)(f2u(x) >> 16); }",
     "static uint16_t trunc16_c(float x) { return (uint16_t)((f2u(x) + 0x8000u) >> 16); }"),
    ("truncation_keeps_15_bits",
     "static uint16_t trunc16_c(float x) { return (uint16_t)(f2u(x) >> 16); }",
     "static uint16_t trunc16_c(float x) { return (uint16_t)((f2u(x) >> 16) & 0xfffeu); }"),
    ("quantiser_ties_away_from_zero",
     "float r = rintf(t);", "float r = roundf(t);"),
    ("quantiser_truncates",
     "float r = rintf(t);", "float r = truncf(t);"),
    ("quantiser_range_128",
     "float inv = 127.0f / scale;", "float inv = 128.0f / scale;"),
    ("quantiser_scale_is_signed_max",
     "float a = fabsf(x[i]);", "float a = x[i];"),
    ("quantiser_no_saturation",
     "if (inv > FLT_MAX) inv = FLT_MAX;", ""),
    ("dequantise_with_scale_not_step",
     "float step = scale / 127.0f;", "float step = scale / 128.0f;"),
    ("quant_blocks_of_2048",
     "#define ORC_QBLOCK 4096u", "#define ORC_QBLOCK 2048u"),
    ("receiver_truncates_its_local_operand",
     "for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i] + mine[i];",
     # (volatile: gcc 11 -O2 folds the plain d(c(x)) round trip inside a conditional back to x)
     "for (size_t i = 0; i < m->len; ++i) { volatile uint16_t h = trunc16_c(mine[i]); "
     "mine[i] = R->tmp[i] + (R->mode == ORC_TRUNC16 ? trunc16_d(h) : mine[i]); }"),
    ("hop_forgets_to_add",
     "for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i] + mine[i];",
     "for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i];"),
    ("hop_subtracts",
     "for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i] + mine[i];",
     "for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i] - mine[i];"),
    ("one_round_too_few",
     "for (int s = 0; s + 1 < p; ++s) orc_ring_reduce_scatter_step(R, s);",
     "for (int s = 0; s + 2 < p; ++s) orc_ring_reduce_scatter_step(R, s);"),
    ("allgather_sends_stale_block",
     "int c = modp(r + 1 - s, p);\n        int to = modp(r + 1, p);", "int c = modp(r - s, p);\n        int to = modp(r + 1, p);"),
    ("update_sign",
     "w[i] = fmaf(-lr, gi, w[i]);", "w[i] = fmaf(lr, gi, w[i]);"),
    ("update_two_roundings",
     "w[i] = fmaf(-lr, gi, w[i]);", "{ volatile float t = lr * gi; w[i] = w[i] - t; }"),
    ("momentum_scales_the_gradient_too",
     "v[i] = fmaf(momentum, v[i], gi);", "v[i] = momentum * (v[i] + gi);"),
    ("momentum_step_uses_gradient_not_velocity",
     "w[i] = fmaf(-lr, v[i], w[i]);", "w[i] = fmaf(-lr, gi, w[i]);"),
    ("grad_scale_ignored",
     "if (grad_scale != 1.0f) gi = gi * grad_scale;", ""),
    ("chunks_not_block_aligned",
     "return (per + ORC_QBLOCK - 1) / ORC_QBLOCK * ORC_QBLOCK;", "return per;"),
    ("hd_halving_distances_ascend",
     "for (int h = p / 2; h >= 1; h /= 2) {               /* halving rounds */",
     "for (int h = 1; h < p; h *= 2) {               /* halving rounds */"),
    ("hd_keeps_the_half_it_should_send",
     "int partner = r ^ h, keep0 = r & ~(h - 1);", "int partner = r ^ h, keep0 = (r & ~(h - 1)) ^ h;"),
    ("hd_receiver_truncates_its_own_partial_sum",
     "for (size_t i = 0; i < hi - lo; ++i) acc[r][lo + i] = acc[r][lo + i] + tmp[i];",
     "for (size_t i = 0; i < hi - lo; ++i) { volatile uint16_t hh = trunc16_c(acc[r][lo + i]); "
     "acc[r][lo + i] = (mode == ORC_TRUNC16 ? trunc16_d(hh) : acc[r][lo + i]) + tmp[i]; }"),
    ("hd_partial_sums_travel_uncompressed",
     "for (size_t i = 0; i < hi - lo; ++i) acc[r][lo + i] = acc[r][lo + i] + tmp[i];",
     "for (size_t i = 0; i < hi - lo; ++i) acc[r][lo + i] = acc[r][lo + i] + acc[partner][lo + i];"),
    ("hd_pairs_neighbours_first",
     "int partner = r ^ h, keep0 = r & ~(h - 1);",
     "int partner = r ^ (p / 2 / h), keep0 = r & ~(h - 1);"),
    ("hd_doubling_takes_the_wrong_blocks",
     "int partner = r ^ d, have0 = partner & ~(d - 1);", "int partner = r ^ d, have0 = r & ~(d - 1);"),
    ("hd_reports_the_ring_round_count",
     "if (counters) { counters[0] = (uint64_t)rounds; counters[1] = sent0; counters[2] = reduced0; }\n    for (int r = 0; r < p; ++r) { free(acc[r]);",
     "if (counters) { counters[0] = (uint64_t)(2 * (p - 1)); counters[1] = sent0; counters[2] = reduced0; }\n    for (int r = 0; r < p; ++r) { free(acc[r]);"),
    ("hd_volume_counts_the_halving_only",
     "if (partner == 0) sent0 += hi - lo;", ""),
    ("direct_adds_in_the_opposite_order",
     "int k = modp(j + d, p);", "int k = modp(j - d, p);"),
    ("direct_contributions_travel_uncompressed",
     "orc_decompress(mode, msg, msg_sc, len, tmp);",
     "for (size_t i = 0; i < len; ++i) tmp[i] = g_local[k][lo + i];"),
    ("direct_owner_compresses_its_own_block_too",
     "for (size_t i = 0; i < len; ++i) P[i] = g_local[j][lo + i];",
     "for (size_t i = 0; i < len; ++i) P[i] = g_local[j][lo + i]; "
     "orc_compress(mode, P, len, msg, msg_sc); orc_decompress(mode, msg, msg_sc, len, P);"),
    ("direct_result_not_compressed_for_the_owner",
     "for (int r = 0; r < p; ++r) {                   /* exchange 2: j -> everyone (and its own copy) */",
     "for (int r = 0; r < p; ++r) { if (r == j && mode == ORC_NONE + 1) { for (size_t i = 0; i < len; ++i) "
     "((uint16_t *)out_payload[r])[lo + i] = (uint16_t)((f2u(P[i]) + 0x8000u) >> 16); continue; }"),
    ("direct_reports_one_round",
     "counters[0] = p > 1 ? 2 : 0;", "counters[0] = p > 1 ? 1 : 0;"),
    ("counters_count_one_direction_only",
     "R->elems_sent[r] += len;\n        R->bytes_sent[r] += nb + 4 * ns;", ""),
]


def build_mutant(tmp_path, name, find, repl):
    text = open(SRC).read()
    assert text.count(find) == 1, f"mutation site for {name} not found exactly once"
    out_c = tmp_path / f"{name}.c"
    out_so = tmp_path / f"{name}.so"
    out_c.write_text(text.replace(find, repl))
    subprocess.check_call(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                           "-mfma", "-w", str(out_c), "-o", str(out_so), "-lm"])
    return str(out_so)


def run_pins(lib_path):
    env = dict(os.environ, PIPESGD_ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PIN_FILES,
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


def test_unmodified_copy_passes(tmp_path):
    lib = build_mutant(tmp_path, "identity", "#define ORC_QBLOCK 4096u", "#define ORC_QBLOCK 4096u")
    res = run_pins(lib)
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, find, repl):
    lib = build_mutant(tmp_path, name, find, repl)
    res = run_pins(lib)
    assert res.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert " failed" in res.stdout or "Error" in res.stdout, res.stdout[-1500:]


def test_oracle_results_do_not_depend_on_the_optimisation_level(tmp_path):
    """The committed oracle is built with -O2.  Build it again with -O0 and -O3
    and require identical bytes from every exported routine on random inputs:
    an optimiser bug in the checker would otherwise go unnoticed."""
    import ctypes as C

    import numpy as np
    outs = []
    for opt in ("-O0", "-O2", "-O3"):
        so = tmp_path / f"orc{opt}.so"
        subprocess.check_call(["gcc", "-std=c11", opt, "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                               "-mfma", "-w", SRC, "-o", str(so), "-lm"])
        code = f"""
import os, sys, hashlib
import numpy as np
sys.path.insert(0, {ROOT!r})
import oracle as orc
from paper_1811_03619_amd import workloads as W
h = hashlib.sha256()
p, n = 4, 4096 * 9 + 777
g = [W.gaussian(n, 1e-3, 5, (0, r, 0, 0)) for r in range(p)]
for r in range(p):
    g[r][::97] = np.float32([0.0, -0.0, 1e-40, 2.5, -1.5, 1e30, 3e-39][r % 7])
for mode in (0, 1, 2):
    for pay, sc in orc.allreduce(mode, g):
        h.update(pay.tobytes()); h.update(b'' if sc is None else sc.tobytes())
    pay, sc = orc.compress(mode, g[0])
    h.update(orc.decompress(mode, pay, sc).tobytes())
    w, v = W.gaussian(n, 1.0, 6), W.gaussian(n, 0.1, 7)
    orc.sgd_update(mode, pay, sc, w, v, 0.01, 0.9, 0.25)
    h.update(w.tobytes()); h.update(v.tobytes())
    orc.sgd_update(mode, pay, sc, w, None, 0.01, 0.0, 1.0)
    h.update(w.tobytes())
print(h.hexdigest())
"""
        env = dict(os.environ, PIPESGD_ORACLE_LIB=str(so))
        res = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                             stderr=subprocess.PIPE, text=True, timeout=300)
        assert res.returncode == 0, res.stderr[-1500:]
        outs.append(res.stdout.strip())
    assert outs[0] == outs[1] == outs[2], outs
