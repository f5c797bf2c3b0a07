"""Mutation check of the oracle's pins (CPU only).

Each case plants one plausible mistake in a *copy* of oracle/alora_oracle.c (a wrong
comparison, a transposed operand, a flipped sign, a dropped term, swapped K/V, an unstable
grouping order ...), builds it, points the oracle's Python wrapper at the broken build and
re-runs the pin suite: at least one pin has to fail.  All planted indexings stay in bounds.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
from test_oracle_pins import PINS

SRC = os.path.join(os.path.dirname(oracle.__file__), "alora_oracle.c")

MUTANTS = {
    "boundary_row_not_adapted": ("int keep_base = pos[t] < start[seg[t]];",
                                 "int keep_base = pos[t] <= start[seg[t]];"),
    "adapter_zero_treated_as_base": ("active[t] = (uint8_t)(aid[t] >= 0 && !keep_base);",
                                     "active[t] = (uint8_t)(aid[t] > 0 && !keep_base);"),
    "start_of_wrong_request": ("int keep_base = pos[t] < start[seg[t]];",
                               "int keep_base = pos[t] < start[0];"),
    "mask_polarity": ("active[t] = (uint8_t)(aid[t] >= 0 && !keep_base);",
                      "active[t] = (uint8_t)(aid[t] >= 0 && keep_base);"),
    "delta_sign": ("yr[n] += d;", "yr[n] -= d;"),
    "A_transposed": ("s[j] += xr[k] * Aa[(size_t)k * r + j];", "s[j] += xr[k] * Aa[(size_t)j * H + k];"),
    "B_transposed": ("d += s[j] * Ba[(size_t)j * N + n];\n                yr[n] += d;",
                     "d += s[j] * Ba[(size_t)n * r + j];\n                yr[n] += d;"),
    "base_W_transposed": ("for (int32_t k = 0; k < H; ++k) acc += xr[k] * W[(size_t)k * N + n];",
                          "for (int32_t k = 0; k < H; ++k) acc += xr[k] * W[(size_t)n * H + k];"),
    "dropped_first_term": ("for (int32_t k = 0; k < H; ++k) {\n            const double xv = xr[k];",
                           "for (int32_t k = 1; k < H; ++k) {\n            const double xv = xr[k];"),
    "dropped_last_rank": ("for (int32_t j = 0; j < r; ++j) d += s[j] * Ba[(size_t)j * N + n];\n                yr[n] += d;",
                          "for (int32_t j = 0; j + 1 < r; ++j) d += s[j] * Ba[(size_t)j * N + n];\n                yr[n] += d;"),
    "delta_on_inactive_rows": ("        if (active[t]) {\n            const double *Aa",
                               "        if (aid[t] >= 0) {\n            const double *Aa"),
    "kv_swapped": ("for (int32_t c = 0; c < Nkv; ++c) kd[c] = yr[Nq + c];",
                   "for (int32_t c = 0; c < Nkv; ++c) kd[c] = yr[Nq + Nkv + c];"),
    "q_shifted": ("q_out[(size_t)t * Nq + c] = yr[c];", "q_out[(size_t)t * Nq + c] = yr[c + 1];"),
    "slot_offset": ("const int64_t off = slot[t] % block_size;", "const int64_t off = (slot[t] + 1) % block_size;"),
    "group_not_stable": ("for (int64_t t = 0; t < T; ++t)\n            if (active[t] && aid[t] == a) perm[n++] = (int32_t)t;",
                         "for (int64_t t = T - 1; t >= 0; --t)\n            if (active[t] && aid[t] == a) perm[n++] = (int32_t)t;"),
    "group_ignores_mask": ("if (active[t]) offsets[aid[t] + 1] += 1;", "if (aid[t] >= 0) offsets[aid[t] + 1] += 1;"),
    "blend_mask_swapped": ("yr[n] = base * m + out * (1.0 - m);", "yr[n] = out * m + base * (1.0 - m);"),
    "var_bias_dropped": ("yt[n] += bias[n];", "yt[n] += 0.0 * bias[n];"),
    "var_bias_only_on_adapted_rows": ("        if (bias)\n            for", "        if (bias && active[tok])\n            for"),
    "var_rank_of_wrong_adapter": ("const int32_t ad = aid[tok], ra = ranks[ad];", "const int32_t ad = aid[tok], ra = ranks[0];"),
    "var_A_pitch_is_common_rank": ("sv[j] += xt[k] * Ar[(size_t)k * ra + j];", "sv[j] += xt[k] * Ar[(size_t)k * ranks[0] + j];"),
    "var_delta_sign": ("yt[n] += dl;", "yt[n] -= dl;"),
    "coords_divisor": ("block[t] = slot[t] / block_size;", "block[t] = slot[t] / (block_size + 1);"),
}


def _run_pins():
    failed = []
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            failed.append(pin.__name__)
    return failed


def test_unmutated_source_passes_all_pins():
    assert _run_pins() == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    needle, repl = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(needle) == 1, f"mutation site for {name} not unique/present"
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(src.replace(needle, repl))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", str(so), str(c)],
                   check=True)
    good = oracle._load()
    bad = ctypes.CDLL(str(so))
    bad.oracle_num_threads.restype = ctypes.c_int
    oracle._lib = bad
    try:
        failed = _run_pins()
    finally:
        oracle._lib = good
    assert failed, f"no pin noticed the planted mistake '{name}'"
