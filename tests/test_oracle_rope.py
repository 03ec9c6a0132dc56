"""Pins for the oracle's rotary encoding: a hand-derived example, complex multiplication (the
definition in its other standard form, through numpy's complex arithmetic), and the properties the
encoding exists for (scores depend on position differences only; norms are kept)."""
import os

import numpy as np

from oracle.rope import rotate, rope_append


def test_hand_example(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "rope_example.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        p, x, y = (part.split() for part in line.split("|"))
        got = rotate(np.array([[[float(v) for v in x]]]), np.array([int(p[0])]), 10000.0)[0, 0]
        assert np.allclose(got, [float(v) for v in y], rtol=0, atol=1e-15), (line, got)
        n += 1
    assert n == 7


def test_equals_complex_multiplication():
    rng = np.random.default_rng(0)
    for D, theta in ((64, 10000.0), (128, 1e6)):
        x = rng.normal(size=(9, 3, D))
        pos = rng.integers(0, 30000, size=9)
        z = x[..., :D // 2] + 1j * x[..., D // 2:]
        freq = theta ** (-np.arange(D // 2) * 2.0 / D)
        w = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
        want = np.concatenate([w.real, w.imag], axis=-1)
        assert np.allclose(rotate(x, pos, theta), want, rtol=0, atol=1e-11)


def test_scores_depend_on_position_difference_only():
    rng = np.random.default_rng(1)
    D, theta = 128, 1e6
    q = rng.normal(size=(1, 1, D))
    k = rng.normal(size=(1, 1, D))
    base = None
    for shift in (0, 1, 17, 4096):
        qr = rotate(q, np.array([25 + shift]), theta)
        kr = rotate(k, np.array([9 + shift]), theta)
        s = float((qr * kr).sum())
        base = s if base is None else base
        assert abs(s - base) < 1e-9
    # and a different difference gives a different score
    s2 = float((rotate(q, np.array([26]), theta) * rotate(k, np.array([9]), theta)).sum())
    assert abs(s2 - base) > 1e-6


def test_norm_kept_and_position_zero_is_identity():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(5, 2, 64))
    pos = np.array([0, 1, 2, 1000, 12345])
    y = rotate(x, pos, 10000.0)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    assert np.array_equal(y[0], x[0])


def test_append_places_rotated_keys_and_plain_values():
    rng = np.random.default_rng(3)
    D, Hq, Hkv, bs, blocks = 64, 4, 2, 16, 5
    k_cache = np.full((blocks, Hkv, bs, D), 7.0)
    v_cache = np.full((blocks, Hkv, bs, D), 7.0)
    q = rng.normal(size=(3, Hq, D))
    k_new = rng.normal(size=(3, Hkv, D))
    v_new = rng.normal(size=(3, Hkv, D))
    pos = np.array([5, 5, 40])
    slots = np.array([3 * bs + 2, 0 * bs + 15, 4 * bs + 0])
    q_rot = rope_append(q, k_new, v_new, pos, slots, k_cache, v_cache, 10000.0)
    assert np.allclose(q_rot, rotate(q, pos, 10000.0))
    for r, (blk, off) in enumerate(((3, 2), (0, 15), (4, 0))):
        assert np.array_equal(v_cache[blk, :, off], v_new[r])
        assert np.allclose(k_cache[blk, :, off], rotate(k_new[r:r + 1], pos[r:r + 1], 10000.0)[0])
    untouched = np.ones((blocks, bs), dtype=bool)
    untouched[[3, 0, 4], [2, 15, 0]] = False
    kt, vt = k_cache.transpose(0, 2, 1, 3), v_cache.transpose(0, 2, 1, 3)   # [blocks][block][Hkv][D]
    assert (kt[untouched] == 7.0).all() and (vt[untouched] == 7.0).all()
