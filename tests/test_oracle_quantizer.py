"""Pins for the oracle's quantizer (Eq. 2, group quantization).  CPU only.

None of these re-types the oracle's threshold formula: they use closed forms,
brute force over the level lattice, a division-based textbook formula, and
invariants that a wrong sign / index / transposed axis would break.
"""
import numpy as np
import pytest

from oracle import kvq_oracle as O


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("bits", [2, 4])
def test_lattice_closed_form(bits):
    # inputs exactly on the lattice z + k*s with power-of-two s: codes are k, round trip exact
    L = (1 << bits) - 1
    for z, s in [(-1.5, 1.0), (0.25, 0.5), (-48.0, 16.0), (3.0, 2.0 ** -6)]:
        k = rng(1).integers(0, L + 1, size=(5, 64))
        k[:, 0] = 0
        k[:, 1] = L                       # make min and max present so range = L*s
        x = (z + k * s).astype(np.float16)
        codes, step, zero = O.quantize_groups(x, bits)
        assert np.array_equal(codes, k)
        assert np.all(step.astype(np.float64) == s) and np.all(zero.astype(np.float64) == z)
        assert np.array_equal(O.dequantize(codes, step, zero), x.astype(np.float64))


@pytest.mark.parametrize("bits", [2, 4])
def test_error_bound_and_extremes(bits):
    g = rng(2)
    x = (g.standard_normal((4000, 32)) * g.choice([0.01, 1.0, 20.0, 200.0], size=(4000, 1))).astype(np.float16)
    codes, step, zero = O.quantize_groups(x, bits)
    L = (1 << bits) - 1
    assert codes.max() <= L
    xh = O.dequantize(codes, step, zero)
    s = step.astype(np.float64)
    normal = s >= 2.0 ** -14
    err = np.abs(xh - x.astype(np.float64))
    assert np.all(err[normal] <= (s[normal] / 2 * (1 + 2.0 ** -9))[:, None])
    # min element -> code 0, max element -> top code (when step > 0)
    am, aM = x.argmin(-1), x.argmax(-1)
    idx = np.arange(x.shape[0])
    assert np.all(codes[idx, am] == 0)
    assert np.all(codes[idx[s > 0], aM[s > 0]] == L)
    assert np.array_equal(zero, x.min(-1))


@pytest.mark.parametrize("bits", [2, 4])
def test_bruteforce_nearest_level(bits):
    # code must be the nearest lattice level to t = fl32(x - mn) (ties to the larger level)
    g = rng(3)
    x = (g.standard_normal((500, 32)) * 3).astype(np.float16)
    codes, step, zero = O.quantize_groups(x, bits)
    L = (1 << bits) - 1
    t = (x.astype(np.float32) - zero.astype(np.float32)[:, None]).astype(np.float64)
    s = step.astype(np.float64)[:, None, None]
    dist = np.abs(t[..., None] - np.arange(L + 1) * s)          # [groups, m, levels]
    best = (L - np.argmin(dist[..., ::-1], axis=-1))              # ties -> larger level
    assert np.array_equal(best, codes)


@pytest.mark.parametrize("bits", [2, 4])
def test_textbook_division_formula(bits):
    # floor((x - mn)/s + 0.5) in fp64, away from near-ties, clamped
    g = rng(4)
    x = (g.standard_normal((2000, 128)) * 2).astype(np.float16)
    codes, step, zero = O.quantize_groups(x, bits)
    L = (1 << bits) - 1
    u = (x.astype(np.float64) - zero.astype(np.float64)[:, None]) / step.astype(np.float64)[:, None]
    far = np.abs(u - np.floor(u) - 0.5) > 1e-3
    ref = np.clip(np.floor(u + 0.5), 0, L)
    assert np.array_equal(ref[far], codes[far].astype(np.float64))


def test_step_is_range_over_levels():
    g = rng(5)
    x = (g.standard_normal((3000, 32)) * 5).astype(np.float16)
    for bits in (2, 4):
        _, step, zero = O.quantize_groups(x, bits)
        true = (x.max(-1).astype(np.float64) - x.min(-1).astype(np.float64)) / ((1 << bits) - 1)
        # fp16 rounding (2^-11) plus one fp32 rounding
        assert np.all(np.abs(step.astype(np.float64) - true) <= true * (2.0 ** -11 + 2.0 ** -22))


def test_constant_and_underflow_groups():
    x = np.full((3, 32), 1.25, np.float16)
    x[1] = 0
    x[2, :16] = np.float16(6e-8)      # subnormal spread: step underflows to 0 or a subnormal
    codes, step, zero = O.quantize_groups(x, 2)
    assert np.all(codes[:2] == 0) and np.all(step[:2] == 0)
    assert np.all(O.dequantize(codes[:2], step[:2], zero[:2]) == x[:2].astype(np.float64))
    if step[2] == 0:
        assert np.all(codes[2] == 0)


@pytest.mark.parametrize("bits", [2, 4])
def test_equivariances(bits):
    g = rng(6)
    x = g.standard_normal((200, 32)).astype(np.float16)
    c0, s0, z0 = O.quantize_groups(x, bits)
    # power-of-two scaling: codes unchanged, step/zero scale
    c1, s1, z1 = O.quantize_groups((x.astype(np.float32) * 8).astype(np.float16), bits)
    assert np.array_equal(c0, c1)
    assert np.array_equal(s1.astype(np.float32), s0.astype(np.float32) * 8)
    assert np.array_equal(z1.astype(np.float32), z0.astype(np.float32) * 8)
    # permutation within the group permutes codes only
    perm = g.permutation(32)
    c2, s2, z2 = O.quantize_groups(np.ascontiguousarray(x[:, perm]), bits)
    assert np.array_equal(c2, c0[:, perm]) and np.array_equal(s2, s0) and np.array_equal(z2, z0)
    # negation reverses the code order
    c3, s3, z3 = O.quantize_groups(-x, bits)
    L = (1 << bits) - 1
    far = np.abs(((x.astype(np.float64) - z0.astype(np.float64)[:, None]) / s0.astype(np.float64)[:, None]) % 1 - 0.5) > 1e-2
    assert np.array_equal(s3, s0)
    assert np.array_equal((L - c3)[far], c0[far])


def test_exhaustive_fp16_against_fixed_params():
    # every finite fp16 value in [mn, mx] against a fixed (mn, step): nearest level in fp64
    allh = np.arange(1 << 16, dtype=np.uint16).view(np.float16)
    allh = allh[np.isfinite(allh)]
    for mn, mx in [(-3.0, 3.0), (0.5, 121.0), (-0.01, 0.02)]:
        vals = allh[(allh >= np.float16(mn)) & (allh <= np.float16(mx))]
        vals = np.concatenate([[np.float16(mn), np.float16(mx)], vals]).astype(np.float16)
        for bits in (2, 4):
            codes, step, zero = O.quantize_groups(vals[None], bits)
            L = (1 << bits) - 1
            t = (vals.astype(np.float32) - np.float32(zero[0])).astype(np.float64)
            u = t / float(step[0])
            ref = np.clip(np.floor(u + 0.5), 0, L)
            far = np.abs(u - np.floor(u) - 0.5) > 1e-6
            assert np.array_equal(ref[far], codes[0][far].astype(np.float64))
            assert np.all(np.diff(codes[0][2:].astype(int)[np.argsort(vals[2:], kind="stable")]) >= 0)


def test_kv_group_axes_and_independence():
    # K parameters are per channel over the G tokens; V parameters per token per channel group
    g = rng(7)
    G, hd, Gv = 32, 128, 32
    k = g.standard_normal((G, hd)).astype(np.float16)
    v = g.standard_normal((G, hd)).astype(np.float16)
    sel = np.zeros(G, bool)
    q0 = O.quantize_kv_group(k, v, sel, 2, Gv)
    assert q0["k_step"].shape == (hd,) and q0["v_step"].shape == (G, hd // Gv)
    # K: channel c's (step, zero, codes) equal a 1-D quantization of that column
    for c in (0, 5, 127):
        cc, ss, zz = O.quantize_groups(np.ascontiguousarray(k[:, c])[None], 2)
        assert np.array_equal(cc[0], q0["k_codes"][:, c]) and ss[0] == q0["k_step"][c] and zz[0] == q0["k_zero"][c]
    # V: changing one token changes only that token's codes / params
    v2 = v.copy(); v2[7] *= np.float16(3)
    q1 = O.quantize_kv_group(k, v2, sel, 2, Gv)
    other = np.arange(G) != 7
    assert np.array_equal(q1["v_codes"][other], q0["v_codes"][other])
    assert np.array_equal(q1["v_step"][other], q0["v_step"][other])
    # K: changing one element changes only its channel
    k2 = k.copy(); k2[3, 40] = np.float16(50)
    q2 = O.quantize_kv_group(k2, v, sel, 2, Gv)
    oc = np.arange(hd) != 40
    assert np.array_equal(q2["k_codes"][:, oc], q0["k_codes"][:, oc])
    assert not np.array_equal(q2["k_codes"][:, 40], q0["k_codes"][:, 40])
    # V channel groups: token 0's group 1 = channels 32..63
    cc, ss, zz = O.quantize_groups(v[0, 32:64][None], 2)
    assert np.array_equal(cc[0], q0["v_codes"][0, 32:64]) and ss[0] == q0["v_step"][0, 1]


def test_zero_minimum_is_stored_as_plus_zero():
    # fp16 has two zeros; the stored zero point of a group whose minimum is zero must be the same
    # pattern whichever of them the group holds (and a negative minimum keeps its sign)
    x = np.array([[0.0, -0.0, 1.0, 2.0], [-0.0, -0.0, -0.0, -0.0], [-0.0, 3.0, 0.0, 1.5], [-1.0, 0.0, -0.0, 2.0]],
                 dtype=np.float16)
    codes, step, zero = O.quantize_groups(x, 2)
    assert zero.view(np.uint16).tolist() == [0x0000, 0x0000, 0x0000, 0xBC00]
    assert codes[1].tolist() == [0, 0, 0, 0] and step[1] == 0
    assert codes[0].tolist() == [0, 0, 2, 3] and codes[2].tolist() == [0, 3, 0, 2]
