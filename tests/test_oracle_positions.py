"""Pins of the position-id and rotary-embedding oracle (oracle/loma_positions.py), CPU only.

Position ids: Eq. 14's closed form and the two purposes Sec. 4.5 states for it; the appendix's arithmetic
(written out here as the listing's range expression evaluated by hand on an example, stored under
tests/golden/); agreement of the training-sample ids with what the generation loop hands out.
Rotary embedding: closed forms (d = 2 is a plane rotation), the frequency ladder, norm preservation, the
relative-position property that defines it, composition of rotations, and a library cross-check with complex
multiplication (numpy's complex exponential: a different route to the same rotation).
"""
import os

import numpy as np
import pytest

from oracle import loma_positions as lp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "position_ids_t2_c3.txt")


def test_eq14_closed_form_and_its_two_purposes():
    for t, c in [(2, 3), (8, 4), (16, 4), (32, 8), (1, 1), (5, 7)]:
        R = t * c
        for i in (0, 1, 5):
            mem = lp.memory_position_ids(i, t, c)
            assert mem[0] == i * R + c - 1 and mem[-1] == i * R + R - 1            # Eq. 14's first and last term
            assert np.all(np.diff(mem) == c) and mem.size == t
            # purpose 2: contiguous with the next chunk's reading zone
            assert mem[-1] + 1 == (i + 1) * R
            # every memory id is an id of its own chunk's reading zone
            assert np.all((mem >= i * R) & (mem < (i + 1) * R))


def test_golden_example_from_the_appendix_arithmetic():
    """t = 2, c = 3 (reading zone of 6): ids worked out by hand from Eq. 14 and from the appendix's
    range(cursor - read_len + c - 1, cursor, c) and range(mem_cursor, mem_cursor + mem_len)."""
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    want = {r[0]: np.array(r[1:], dtype=np.int64) for r in rows}
    assert np.array_equal(lp.sample_position_ids(2, 3, 2, lp.INTERMITTENT), want["sample_intermittent"])
    assert np.array_equal(lp.sample_position_ids(2, 3, 2, lp.CONTIGUOUS), want["sample_contiguous"])
    assert np.array_equal(lp.compress_position_ids(12, 2, 3, 1, lp.INTERMITTENT), want["compress_cursor12_intermittent"])
    assert np.array_equal(lp.compress_position_ids(12, 2, 3, 1, lp.CONTIGUOUS), want["compress_cursor12_contiguous"])


@pytest.mark.parametrize("ptype", [lp.INTERMITTENT, lp.CONTIGUOUS])
@pytest.mark.parametrize("t,c,n", [(2, 3, 4), (16, 4, 3), (4, 1, 5)])
def test_training_ids_equal_generation_ids(t, c, n, ptype):
    """Walking the generation loop (cursor advances by real tokens only, compression after every t*c of them)
    hands every reading and memory token the id it has in the training sample."""
    R, s = t * c, t * (2 * c + 1)
    sample = lp.sample_position_ids(t, c, n, ptype)
    cursor = 0
    for i in range(n):
        got = lp.generation_position_ids(cursor, R)
        assert np.array_equal(got, sample[i * s: i * s + R])
        assert np.array_equal(got, np.arange(i * R, (i + 1) * R))                # purpose 1: original ids preserved
        cursor += R
        mem = lp.compress_position_ids(cursor, t, c, i, ptype)
        assert np.array_equal(mem, sample[i * s + R: i * s + R + t])
        assert np.array_equal(mem, lp.memory_position_ids(i, t, c, ptype))
        # repetition tokens carry the ids of the tokens they reproduce
        assert np.array_equal(sample[i * s + R + t: (i + 1) * s], np.arange(i * R, (i + 1) * R))
    with pytest.raises(ValueError):
        lp.compress_position_ids(R - 1, t, c, 0, ptype)
    with pytest.raises(ValueError):
        lp.memory_position_ids(0, t, c, "other")


def test_rope_closed_forms():
    # d = 2: one pair, frequency theta^0 = 1: a rotation of the plane by `pos` radians
    x = np.array([[1.0, 0.0], [0.0, 1.0], [3.0, -2.0]])
    y = lp.rope_rotate(x, [1, 1, 2])
    np.testing.assert_allclose(y[0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    np.testing.assert_allclose(y[1], [-np.sin(1.0), np.cos(1.0)], atol=1e-15)
    np.testing.assert_allclose(y[2], [3 * np.cos(2.0) + 2 * np.sin(2.0), -2 * np.cos(2.0) + 3 * np.sin(2.0)], atol=1e-15)
    # position 0 is the identity
    z = np.arange(24.0).reshape(3, 8)
    assert np.array_equal(lp.rope_rotate(z, [0, 0, 0]), z)
    # the frequency ladder: d = 4, theta = 10000 -> pairs (0,2) at 1 rad/position, (1,3) at 0.01 rad/position
    a = lp.rope_angles([7], 4, 10000.0)
    np.testing.assert_allclose(a, [[7.0, 0.07]], rtol=1e-15)
    a = lp.rope_angles([3], 128, 10000.0)
    np.testing.assert_allclose(a[0, 32], 3 * 10000.0 ** -0.5, rtol=1e-15)         # element 32 of 64: theta^(-1/2)
    # element i pairs with i + d/2 (not with i + 1): only the pair (1, 3) moves when x is zero elsewhere
    e = np.zeros((1, 4)); e[0, 1] = 1.0
    y = lp.rope_rotate(e, [100])
    assert y[0, 0] == 0 and y[0, 2] == 0
    np.testing.assert_allclose([y[0, 1], y[0, 3]], [np.cos(1.0), np.sin(1.0)], atol=1e-13)


def test_rope_properties_and_complex_cross_check():
    rng = np.random.default_rng(94860014)
    d, L = 64, 9
    q, k = rng.standard_normal((2, 3, L, d)), rng.standard_normal((2, 3, L, d))
    pos = np.array([0, 1, 5, 17, 100, 1023, 4096, 70001, 131071])
    qr, kr = lp.rope_rotate(q, pos), lp.rope_rotate(k, pos)
    # norms are preserved
    np.testing.assert_allclose(np.linalg.norm(qr, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-12)
    # scores depend on the position difference only: <R(m) q, R(n) k> = <R(m - n) q, k>
    for a in range(L):
        for b in range(a + 1):
            lhs = np.einsum("bhd,bhd->bh", qr[:, :, a], kr[:, :, b])
            rel = lp.rope_rotate(q[:, :, a:a + 1], [pos[a] - pos[b]])[:, :, 0]
            np.testing.assert_allclose(lhs, np.einsum("bhd,bhd->bh", rel, k[:, :, b]), atol=1e-9)
    # rotations compose: R(a) R(b) = R(a + b)
    twice = lp.rope_rotate(lp.rope_rotate(q, pos), pos[::-1].copy())
    np.testing.assert_allclose(twice, lp.rope_rotate(q, pos + pos[::-1]), atol=1e-9)
    # library route: (x_i + j x_{i+d/2}) * exp(j a_i) with numpy's complex arithmetic
    theta = 500000.0
    inv = theta ** (-np.arange(0, d, 2) / d)
    z = (q[..., : d // 2] + 1j * q[..., d // 2:]) * np.exp(1j * pos[:, None] * inv[None, :])
    np.testing.assert_allclose(lp.rope_rotate(q, pos, theta), np.concatenate([z.real, z.imag], axis=-1), atol=1e-9)


def test_round_to_storage_types():
    """One rounding, fp64 -> storage type, to nearest even: checked against the definition (no representable
    neighbour is nearer) and, away from ties, against torch's conversion (which goes through fp32)."""
    import torch
    rng = np.random.default_rng(5)
    x = rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))
    x[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -(1.0 + 2.0 ** -8 + 2.0 ** -30)]   # two ties, two near-ties
    bits = lp.round_to(x, "bf16")
    val = lambda b: (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = val(bits)
    assert got[0] == 1.0 and got[1] == 1.015625 and got[2] == 1.0 and got[3] == -1.0078125
    for nb in (bits + np.uint16(1), bits - np.uint16(1)):         # the neighbours in magnitude
        d_got, d_nb = np.abs(x - got), np.abs(x - val(nb))
        assert np.all(d_got <= d_nb)
        ties = d_got == d_nb
        assert np.all((bits[ties] & 1) == 0)                      # ties go to the even significand
    want = torch.from_numpy(x[4:]).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got[4:].astype(np.float32), want)
    assert np.array_equal(lp.round_to(x, "f32"), x.astype(np.float32))
