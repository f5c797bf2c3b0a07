"""Pins of the attention oracle (oracle/attention.py), CPU only.

The paper states causal softmax attention in words (Sec. 2.1); the pins fix the oracle to things
that are not the oracle itself: a library routine on the special case it covers, closed forms,
a plain-Python brute force, and invariances of the paged layout.  The second half plants one
plausible mistake at a time in a copy of the oracle's source and requires some pin to fail.
"""
import math
import os
import types

import numpy as np
import pytest
import torch

import oracle
from oracle import attention as att

SRC = os.path.join(os.path.dirname(oracle.__file__), "attention.py")


def _case(seed, n_seq=3, hq=4, hkv=2, d=8, bs=4, max_len=19, extra_blocks=3):
    """Random paged cache: sequences of ragged length, physical blocks a permutation, every sequence's
    last `n_rows` positions are query rows."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, n_seq)
    nb = [(int(l) + bs - 1) // bs for l in lens]
    n_blocks = sum(nb) + extra_blocks
    perm = rng.permutation(n_blocks)
    max_blocks = max(nb) + 1
    bt = np.full((n_seq, max_blocks), -1, np.int32)
    o = 0
    for s in range(n_seq):
        bt[s, :nb[s]] = perm[o:o + nb[s]]
        o += nb[s]
    kc = rng.standard_normal((n_blocks * bs, hkv * d))
    vc = rng.standard_normal((n_blocks * bs, hkv * d))
    seq, pos = [], []
    for s in range(n_seq):
        n_rows = int(rng.integers(1, min(4, lens[s]) + 1))
        for p in range(lens[s] - n_rows, lens[s]):
            seq.append(s)
            pos.append(p)
    seq, pos = np.asarray(seq, np.int32), np.asarray(pos, np.int32)
    q = rng.standard_normal((len(seq), hq * d))
    return dict(q=q, kc=kc, vc=vc, bt=bt, seq=seq, pos=pos, bs=bs, hq=hq, hkv=hkv, d=d, lens=lens)


def _run(mod, c, **kw):
    return mod.paged_attention(c["q"], c["kc"], c["vc"], c["bt"], c["seq"], c["pos"], c["bs"], c["hq"], c["hkv"], c["d"], **kw)


# ----------------------------------------------------------------------------------------------
# pins (each takes the module under test so that the mutation check can re-run them)
# ----------------------------------------------------------------------------------------------
def pin_library_routine_on_a_contiguous_sequence(mod=att):
    """One sequence whose every position is a query row, identity block table: the library's causal
    scaled-dot-product attention (fp64, CPU) computes the same thing, head by head."""
    rng = np.random.default_rng(11)
    n, hq, hkv, d, bs = 13, 6, 2, 16, 4
    q = rng.standard_normal((n, hq * d))
    kc = rng.standard_normal((16, hkv * d))
    vc = rng.standard_normal((16, hkv * d))
    bt = np.arange(4, dtype=np.int32)[None, :]
    got = mod.paged_attention(q, kc, vc, bt, np.zeros(n, np.int32), np.arange(n, dtype=np.int32), bs, hq, hkv, d)
    tq = torch.from_numpy(q).reshape(n, hq, d).permute(1, 0, 2)[None]                      # [1, hq, n, d]
    tk = torch.from_numpy(kc[:n]).reshape(n, hkv, d).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    tv = torch.from_numpy(vc[:n]).reshape(n, hkv, d).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0]  # [hq, n, d]
    ref = ref.permute(1, 0, 2).reshape(n, hq * d).numpy()
    assert np.abs(got - ref).max() <= 1e-12


def pin_plain_python_brute_force(mod=att):
    c = _case(5, n_seq=2, hq=2, hkv=1, d=3, bs=2, max_len=5)
    got = _run(mod, c)
    for i in range(len(c["seq"])):
        s, p = int(c["seq"][i]), int(c["pos"][i])
        for h in range(c["hq"]):
            g = h // (c["hq"] // c["hkv"])
            scores = []
            for j in range(p + 1):
                slot = int(c["bt"][s][j // c["bs"]]) * c["bs"] + j % c["bs"]
                dot = 0.0
                for e in range(c["d"]):
                    dot += c["q"][i][h * c["d"] + e] * c["kc"][slot][g * c["d"] + e]
                scores.append(dot / math.sqrt(c["d"]))
            z = sum(math.exp(x) for x in scores)
            for e in range(c["d"]):
                val = 0.0
                for j in range(p + 1):
                    slot = int(c["bt"][s][j // c["bs"]]) * c["bs"] + j % c["bs"]
                    val += math.exp(scores[j]) / z * c["vc"][slot][g * c["d"] + e]
                assert abs(got[i][h * c["d"] + e] - val) <= 1e-12


def pin_equal_keys_give_the_mean_of_the_values(mod=att):
    c = _case(7)
    c["kc"][:] = c["kc"][0]           # every cached key row the same: all scores equal
    got = _run(mod, c)
    for i in range(len(c["seq"])):
        p = int(c["pos"][i])
        slots = att.context_slots(c["bt"][c["seq"][i]], p + 1, c["bs"])
        mean = c["vc"][slots].mean(axis=0)                       # [hkv*d]
        for h in range(c["hq"]):
            g = h // (c["hq"] // c["hkv"])
            assert np.abs(got[i, h * c["d"]:(h + 1) * c["d"]] - mean[g * c["d"]:(g + 1) * c["d"]]).max() <= 1e-12


def pin_two_positions_closed_form(mod=att):
    """Position 1 attending to two keys: weights are the logistic function of the scaled score gap."""
    d, bs = 4, 2
    q = np.array([[0.0] * d, [1.0, 2.0, -1.0, 0.5]])
    kc = np.array([[0.3, -0.2, 0.1, 0.7], [1.1, 0.4, -0.6, 0.2]])
    vc = np.array([[1.0, 2.0, 3.0, 4.0], [-1.0, 0.5, 0.0, 8.0]])
    bt = np.array([[0]], np.int32)
    got = mod.paged_attention(q, kc, vc, bt, np.zeros(2, np.int32), np.array([0, 1], np.int32), bs, 1, 1, d)
    assert np.abs(got[0] - vc[0]).max() <= 1e-15              # a single key: weight 1
    gap = (q[1] @ kc[1] - q[1] @ kc[0]) / 2.0                 # 1/sqrt(4)
    w1 = 1.0 / (1.0 + math.exp(-gap))
    assert np.abs(got[1] - ((1 - w1) * vc[0] + w1 * vc[1])).max() <= 1e-14
    # explicit scale
    got2 = mod.paged_attention(q, kc, vc, bt, np.zeros(2, np.int32), np.array([0, 1], np.int32), bs, 1, 1, d, scale=0.125)
    w1 = 1.0 / (1.0 + math.exp(-(q[1] @ kc[1] - q[1] @ kc[0]) * 0.125))
    assert np.abs(got2[1] - ((1 - w1) * vc[0] + w1 * vc[1])).max() <= 1e-14


def pin_one_dominant_key_selects_its_value(mod=att):
    c = _case(9, n_seq=1, hq=2, hkv=2, d=8, max_len=12)
    i = len(c["seq"]) - 1
    p = int(c["pos"][i])
    slots = att.context_slots(c["bt"][0], p + 1, c["bs"])
    for target in (0, p // 2, p):
        kc = c["kc"] * 1e-3
        for h in range(2):
            kc[slots[target], h * 8:(h + 1) * 8] = 400.0 * c["q"][i, h * 8:(h + 1) * 8]
        got = mod.paged_attention(c["q"], kc, c["vc"], c["bt"], c["seq"], c["pos"], c["bs"], 2, 2, 8)
        assert np.abs(got[i] - c["vc"][slots[target]]).max() <= 1e-9


def pin_future_and_foreign_slots_are_never_read_and_the_own_position_is(mod=att):
    c = _case(13)
    base = _run(mod, c)
    used = np.zeros(c["kc"].shape[0], bool)
    for s in range(len(c["lens"])):
        used[att.context_slots(c["bt"][s], int(c["lens"][s]), c["bs"])] = True
    # poison everything outside the contexts (spare blocks, tails of last blocks) ...
    kc, vc = c["kc"].copy(), c["vc"].copy()
    kc[~used] = np.nan
    vc[~used] = np.nan
    c2 = dict(c, kc=kc, vc=vc)
    assert np.array_equal(_run(mod, c2), base)
    # ... and, for a row that is not the last of its sequence, the positions after it
    for i in range(len(c["seq"])):
        s, p = int(c["seq"][i]), int(c["pos"][i])
        if p + 1 < c["lens"][s]:
            later = att.context_slots(c["bt"][s], int(c["lens"][s]), c["bs"])[p + 1:]
            kc3, vc3 = c["kc"].copy(), c["vc"].copy()
            kc3[later] = np.nan
            vc3[later] = np.nan
            got = mod.paged_attention(c["q"], kc3, vc3, c["bt"], c["seq"], c["pos"], c["bs"], c["hq"], c["hkv"], c["d"], rows=np.array([i]))
            assert np.array_equal(got[0], base[i])
            # its own position does count
            own = att.context_slots(c["bt"][s], p + 1, c["bs"])[p]
            vc4 = c["vc"].copy()
            vc4[own] += 1.0
            got = mod.paged_attention(c["q"], c["kc"], vc4, c["bt"], c["seq"], c["pos"], c["bs"], c["hq"], c["hkv"], c["d"], rows=np.array([i]))
            assert np.abs(got[0] - base[i]).min() > 1e-6
            break
    else:
        raise AssertionError("case has no interior row")


def pin_physical_placement_does_not_matter(mod=att):
    c = _case(17)
    base = _run(mod, c)
    n_blocks = c["kc"].shape[0] // c["bs"]
    rng = np.random.default_rng(3)
    new_of = rng.permutation(n_blocks)                 # old block b moves to new_of[b]
    kc, vc = np.empty_like(c["kc"]), np.empty_like(c["vc"])
    for b in range(n_blocks):
        kc[new_of[b] * c["bs"]:(new_of[b] + 1) * c["bs"]] = c["kc"][b * c["bs"]:(b + 1) * c["bs"]]
        vc[new_of[b] * c["bs"]:(new_of[b] + 1) * c["bs"]] = c["vc"][b * c["bs"]:(b + 1) * c["bs"]]
    bt = np.where(c["bt"] >= 0, new_of[np.maximum(c["bt"], 0)], -1).astype(np.int32)
    got = _run(mod, dict(c, kc=kc, vc=vc, bt=bt))
    assert np.abs(got - base).max() <= 1e-13


def pin_query_heads_read_their_own_kv_head(mod=att):
    c = _case(19, hq=6, hkv=3, d=4)
    vc = np.empty_like(c["vc"])
    for g in range(3):
        vc[:, g * 4:(g + 1) * 4] = float(g + 1)       # V of K/V head g is the constant g+1
    got = _run(mod, dict(c, vc=vc))
    want = np.repeat(np.array([1.0, 1.0, 2.0, 2.0, 3.0, 3.0]), 4)
    assert np.abs(got - want[None, :]).max() <= 1e-13
    # and the scores use that head's keys: scaling the keys of head 0 only moves query heads 0 and 1
    base = _run(mod, c)
    kc = c["kc"].copy()
    kc[:, 0:4] *= 3.0
    got = _run(mod, dict(c, kc=kc))
    multi = c["pos"] > 0
    assert np.abs(got[multi, :8] - base[multi, :8]).max() > 1e-6
    assert np.array_equal(got[:, 8:], base[:, 8:])


def pin_softmax_shift_and_value_linearity(mod=att):
    c = _case(23)
    base = _run(mod, c)
    # adding a vector orthogonal to nothing in particular to all keys of a head shifts every score of a
    # query by the same amount: no change
    kc = c["kc"].copy()
    shift = np.random.default_rng(1).standard_normal(c["hkv"] * c["d"])
    kc += shift[None, :]
    assert np.abs(_run(mod, dict(c, kc=kc)) - base).max() <= 1e-11
    # the output is linear in V, and a constant added to V is added to the output (weights sum to 1)
    assert np.abs(_run(mod, dict(c, vc=2.0 * c["vc"] + 5.0)) - (2.0 * base + 5.0)).max() <= 1e-12


PINS = [pin_library_routine_on_a_contiguous_sequence, pin_plain_python_brute_force,
        pin_equal_keys_give_the_mean_of_the_values, pin_two_positions_closed_form,
        pin_one_dominant_key_selects_its_value, pin_future_and_foreign_slots_are_never_read_and_the_own_position_is,
        pin_physical_placement_does_not_matter, pin_query_heads_read_their_own_kv_head,
        pin_softmax_shift_and_value_linearity]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin()


# ----------------------------------------------------------------------------------------------
# planted mistakes
# ----------------------------------------------------------------------------------------------
MUTANTS = {
    "own_position_excluded": ("slots = context_slots(block_tables[int(token_seq_ids[t])], p + 1, block_size)\n        K = k_cache[slots].reshape(p + 1,",
                              "slots = context_slots(block_tables[int(token_seq_ids[t])], max(p, 1), block_size)\n        K = k_cache[slots].reshape(max(p, 1),"),
    "no_scale": ("scale = 1.0 / np.sqrt(float(head_dim))", "scale = 1.0"),
    "scale_by_d_not_sqrt_d": ("scale = 1.0 / np.sqrt(float(head_dim))", "scale = 1.0 / float(head_dim)"),
    "explicit_scale_ignored": ("    if scale is None:\n", "    if True:\n"),
    "kv_head_modulo_not_division": ("g = h // group", "g = h % n_kv_heads"),
    "values_of_head_zero": ("out[i, h * head_dim:(h + 1) * head_dim] = w @ V[:, g, :]", "out[i, h * head_dim:(h + 1) * head_dim] = w @ V[:, 0, :]"),
    "not_normalised": ("w = w / w.sum()", "w = w / 1.0"),
    "score_sign": ("score = scale * (K[:, g, :] @ qh)", "score = -scale * (K[:, g, :] @ qh)"),
    "slot_ignores_offset": (".astype(np.int64) * block_size + j % block_size", ".astype(np.int64) * block_size + 0 * (j % block_size)"),
    "table_of_sequence_zero": ("block_tables[int(token_seq_ids[t])]", "block_tables[0]"),
    "block_index_off_by_one": ("block_table_row[j // block_size]", "block_table_row[(j + 1) // block_size]"),
    "k_and_v_swapped": ("V = v_cache[slots].reshape(p + 1, n_kv_heads, head_dim)", "V = k_cache[slots].reshape(p + 1, n_kv_heads, head_dim)"),
    "query_of_head_zero": ("qh = q[t, h * head_dim:(h + 1) * head_dim]", "qh = q[t, 0:head_dim]"),
}


def _load_mutant(needle, repl):
    src = open(SRC).read()
    assert src.count(needle) == 1, "mutation site not unique/present"
    mod = types.ModuleType("attention_mutant")
    exec(compile(src.replace(needle, repl), "attention_mutant.py", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    mod = _load_mutant(*MUTANTS[name])
    failed = []
    for pin in PINS:
        try:
            pin(mod)
        except (AssertionError, IndexError, ValueError):
            failed.append(pin.__name__)
    assert failed, f"no pin notices the planted mistake '{name}'"
