"""Pins of the rotary-embedding oracle (oracle/rope.py) against things it does not compute itself: complex
multiplication, closed forms, the invariants of a rotation, and planted mistakes."""
import numpy as np
import pytest

from oracle import rope as orope
from paper_2512_17910_amd import workloads as wl


def _case(seed=0, R=7, hq=3, hkv=2, D=8, max_pos=50):
    rng = np.random.default_rng(seed)
    y = rng.standard_normal((R, (hq + 2 * hkv) * D))
    pos = rng.integers(0, max_pos, R)
    cos, sin = wl.rope_table(max_pos, D)
    return y, pos, cos.astype(np.float64), sin.astype(np.float64), hq, hkv, D


def _pin_complex(fn):
    y, pos, cos, sin, hq, hkv, D = _case()
    out = fn(y, pos, cos, sin, hq, hkv, D)
    for r in range(y.shape[0]):
        for h in range(hq + hkv):
            for i in range(D // 2):
                z = complex(y[r, h * D + i], y[r, h * D + i + D // 2]) * complex(cos[pos[r], i], sin[pos[r], i])
                assert abs(out[r, h * D + i] - z.real) < 1e-14 and abs(out[r, h * D + i + D // 2] - z.imag) < 1e-14
    assert np.array_equal(out[:, (hq + hkv) * D:], y[:, (hq + hkv) * D:])          # v untouched


def _pin_quarter_turn(fn):
    # D = 2, one q head, one k head, one v head: angle pi/2 sends (1, 0) to (0, 1) and (0, 1) to (-1, 0)
    y = np.array([[1.0, 0.0, 0.0, 1.0, 5.0, 6.0]])
    out = fn(y, [0], np.array([[0.0]]), np.array([[1.0]]), 1, 1, 2)
    assert np.array_equal(out, np.array([[0.0, 1.0, -1.0, 0.0, 5.0, 6.0]]))


def _pin_identity_and_norms(fn):
    y, pos, cos, sin, hq, hkv, D = _case(1)
    assert np.array_equal(fn(y, np.zeros(len(pos), int), cos, sin, hq, hkv, D), y)
    out = fn(y, pos, cos, sin, hq, hkv, D)
    heads = lambda a: a[:, :(hq + hkv) * D].reshape(len(pos), hq + hkv, D)
    # fp32 table entries: cos^2 + sin^2 = 1 to 1e-7
    assert np.allclose(np.linalg.norm(heads(out), axis=2), np.linalg.norm(heads(y), axis=2), rtol=2e-7)


def _pin_distance_only(fn):
    """<R_m q, R_n k> = <R_(m-n) q, k>: the property the embedding exists for (exact cos/sin in fp64)."""
    rng = np.random.default_rng(2)
    D, max_pos = 16, 64
    i = np.arange(D // 2)
    ang = np.arange(max_pos)[:, None] * 10000.0 ** (-2.0 * i / D)[None, :]
    cos, sin = np.cos(ang), np.sin(ang)
    q, k = rng.standard_normal(D), rng.standard_normal(D)
    row = lambda v: np.concatenate([v, v, v])[None, :]            # one q head, one k head, one v head
    rot = lambda v, p: fn(row(v), [p], cos, sin, 1, 1, D)[0, :D]
    for m, n in [(5, 3), (40, 17), (63, 63), (9, 0)]:
        assert abs(rot(q, m) @ rot(k, n) - rot(q, m - n) @ k) < 1e-12
    # and turning by m then by n is turning by m + n
    twice = fn(row(rot(q, 7)), [11], cos, sin, 1, 1, D)[0, :D]
    assert np.allclose(twice, rot(q, 18), atol=1e-13)


def _pin_no_mixing(fn):
    y, pos, cos, sin, hq, hkv, D = _case(3)
    base = fn(y, pos, cos, sin, hq, hkv, D)
    y2 = y.copy()
    y2[2, D:2 * D] += 1.0                                          # head 1 of row 2
    out = fn(y2, pos, cos, sin, hq, hkv, D)
    diff = out != base
    assert diff[2, D:2 * D].any() and not np.delete(diff, 2, axis=0).any()
    assert not diff[2, :D].any() and not diff[2, 2 * D:].any()


PINS = [_pin_complex, _pin_quarter_turn, _pin_identity_and_norms, _pin_distance_only, _pin_no_mixing]


@pytest.mark.parametrize("pin", PINS)
def test_pin(pin):
    pin(orope.rope_rows)


MISTAKES = [
    ("a * c - b * s", "a * c + b * s"),
    ("b * c + a * s", "b * c - a * s"),
    ("c, s = cos[p], sin[p]", "c, s = sin[p], cos[p]"),
    ("p = int(positions[r])", "p = int(positions[0])"),
    ("for h in range(n_q_heads + n_kv_heads):", "for h in range(n_q_heads):"),
    ("for h in range(n_q_heads + n_kv_heads):", "for h in range(n_q_heads + 2 * n_kv_heads):"),
    ("b = y[r, lo + half:lo + head_dim]", "b = y[r, lo + half:lo + head_dim][::-1]"),
    ("lo = h * head_dim", "lo = h * half"),
]


@pytest.mark.parametrize("old,new", MISTAKES)
def test_planted_mistakes_fail_a_pin(old, new):
    import inspect
    src = inspect.getsource(orope)
    assert src.count(old) == 1
    ns = {}
    exec(compile(src.replace(old, new), "mutant", "exec"), ns)
    caught = 0
    for pin in PINS:
        try:
            pin(ns["rope_rows"])
        except (AssertionError, IndexError, ValueError):
            caught += 1
    assert caught >= 1
