"""Pins of the oracle's value rotation (appendix ablation "Value Rotation": V_tn = V_t e^{i eps n}) on the CPU:
closed forms of a plane rotation, the group law, and the same product written with numpy's complex numbers."""
import numpy as np

import oracle
from paper_2402_11131_amd import synth


def _v(seed, B=2, T=5, gamma=3, Hkv=2, D=8):
    rng = synth.rng_for(seed)
    v = rng.standard_normal((B, T * (1 + gamma), Hkv, D)).astype(np.float32)
    return v, T, gamma


def test_zero_angle_copies_the_main_row_and_main_rows_pass_through():
    v, T, gamma = _v(1)
    out = oracle.value_rotate(v, T, gamma, 0.0)
    assert np.array_equal(out[:, :T], v[:, :T].astype(np.float64))
    for i in range(T):
        for n in range(1, gamma + 1):
            assert np.array_equal(out[:, T + i * gamma + n - 1], v[:, i].astype(np.float64))


def test_quarter_turn_maps_re_im_to_minus_im_re():
    v, T, gamma = _v(2, gamma=1)
    out = oracle.value_rotate(v, T, gamma, np.pi / 2)
    for i in range(T):
        s = out[:, T + i]
        assert np.allclose(s[..., 0::2], -v[:, i, :, 1::2], atol=1e-15 * 10, rtol=0)
        assert np.allclose(s[..., 1::2], v[:, i, :, 0::2], atol=1e-15 * 10, rtol=0)


def test_every_pair_keeps_its_length_and_turns_by_eps_times_n():
    v, T, gamma = _v(3)
    eps = 0.137
    out = oracle.value_rotate(v, T, gamma, eps)
    for i in range(T):
        z0 = v[:, i, :, 0::2].astype(np.float64) + 1j * v[:, i, :, 1::2].astype(np.float64)
        for n in range(1, gamma + 1):
            s = out[:, T + i * gamma + n - 1]
            z = s[..., 0::2] + 1j * s[..., 1::2]
            assert np.allclose(np.abs(z), np.abs(z0), rtol=1e-14)
            turn = np.angle(z * np.conj(z0))                     # angle between the two, in (-pi, pi]
            assert np.allclose(turn, eps * n, atol=1e-12)


def test_equals_numpy_complex_product():
    v, T, gamma = _v(4, B=3, T=7, gamma=4, Hkv=3, D=16)
    eps = np.pi / (2 * 4100)                                     # the paper's upper end for N = 4096 + 4
    out = oracle.value_rotate(v, T, gamma, eps)
    for i in range(T):
        z0 = v[:, i, :, 0::2].astype(np.float64) + 1j * v[:, i, :, 1::2].astype(np.float64)
        for n in range(1, gamma + 1):
            z = z0 * np.exp(1j * eps * n)
            s = out[:, T + i * gamma + n - 1]
            assert np.allclose(s[..., 0::2], z.real, rtol=1e-14, atol=1e-300)
            assert np.allclose(s[..., 1::2], z.imag, rtol=1e-14, atol=1e-300)


def test_group_law_stream_n_is_stream_one_applied_n_times():
    # values on a grid of 1/8 so that feeding a rotated row back in stays close to exact; a rotation by eps of the
    # (rounded to fp32) stream-1 row equals stream 2 up to that rounding
    v, T, gamma = _v(5, gamma=2)
    eps = 0.3
    out = oracle.value_rotate(v, T, gamma, eps)
    again = v.copy()
    for i in range(T):
        again[:, i] = out[:, T + i * gamma].astype(np.float32)   # stream 1 of node i as the new main row
    out2 = oracle.value_rotate(again, T, gamma, eps)
    for i in range(T):
        assert np.allclose(out2[:, T + i * gamma], out[:, T + i * gamma + 1], atol=1e-6)


def test_a_stream_row_depends_on_its_own_nodes_main_row_only():
    v, T, gamma = _v(6)
    base = oracle.value_rotate(v, T, gamma, 0.2)
    w = v.copy()
    w[:, T:] = np.nan                                            # what the stream rows held before is never read
    w[:, 2] += 1.0                                               # another node's main row changes
    out = oracle.value_rotate(w, T, gamma, 0.2)
    assert np.isfinite(out).all()
    for i in range(T):
        rows = slice(T + i * gamma, T + (i + 1) * gamma)
        assert np.array_equal(out[:, rows], base[:, rows]) == (i != 2)
