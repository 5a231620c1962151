"""Pins of the oracle's per-step Value schedule (the comparison schedule of the paper's
Experiments, "Details": Keys compressed every G steps, Values at each step).

The quantizer itself is pinned in test_oracle_quantizer.py.  What is pinned here is the schedule:
which tokens are quantized at which context length, that the stored codes do not depend on the
schedule, and that the attention is plain softmax attention over the rows the schedule defines."""
import numpy as np
import pytest
import torch

from oracle import kvq_oracle as O


def _rows(seed, n, hd=128):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((n, hd)).astype(np.float16)
    V = rng.standard_normal((n, hd)).astype(np.float16)
    K[:, [3, 40, 77, 101]] *= 20
    return K, V


@pytest.mark.parametrize("bits,G,Gv,R", [(2, 32, 32, 128), (4, 32, 64, 40), (2, 64, 128, 1), (2, 128, 32, 32)])
def test_stored_codes_do_not_depend_on_the_schedule(bits, G, Gv, R):
    """Token-wise Value groups involve one token only: stepping token by token through the per-step
    schedule leaves, below n_quant, exactly the codes, steps and zeros of the every-G-steps schedule
    without tracing; and the Values beyond are those of the tokens older than R, no more, no fewer."""
    n = 3 * G + R + 17
    K, V = _rows(1, n)
    per = O.PerStepValueUnit(128, bits, G, Gv)
    ref = O.UnitState(128, bits, G, Gv, 0, 0)
    for m in range(1, n + 1):
        per.advance_to(K, V, m, R)
        nq = G * ((m - R) // G) if m >= R + G else 0
        while ref.n_quant < nq:
            ref.append_group(K[ref.n_quant:ref.n_quant + G], V[ref.n_quant:ref.n_quant + G])
        assert per.n_quant == nq
        assert per.n_quant_v == max(0, m - R)
        for name in ("k_codes", "k_step", "k_zero"):
            assert np.array_equal(getattr(per, name).view(np.uint8 if name == "k_codes" else np.uint16),
                                  getattr(ref, name).view(np.uint8 if name == "k_codes" else np.uint16)), name
        for name in ("v_codes", "v_step", "v_zero"):
            a = getattr(per, name)[:nq]
            assert np.array_equal(a.view(np.uint8 if name == "v_codes" else np.uint16),
                                  getattr(ref, name).view(np.uint8 if name == "v_codes" else np.uint16)), name
    pa, pb = O.packed_unit(per), O.packed_unit(ref)
    for name in pa:
        assert np.array_equal(pa[name].view(np.uint8), pb[name].view(np.uint8)), name


@pytest.mark.parametrize("bits,Gv", [(2, 32), (4, 32), (2, 128)])
def test_window_boundary_and_error_bound(bits, Gv):
    """The last R tokens keep their Values bit for bit; every older token's Value is a level of its
    own group: within half a step (plus the fp16 rounding of the level) of the original, equal to it
    at the group's minimum, and not the original row."""
    G, R, n = 32, 48, 150
    K, V = _rows(2, n)
    st = O.PerStepValueUnit(128, bits, G, Gv)
    st.advance_to(K, V, n, R)
    nq = st.n_quant
    _, Veff = st.effective_rows(K[nq:n], V[nq:n])
    assert Veff.shape == (n, 128)
    assert np.array_equal(Veff[n - R:], V[n - R:].astype(np.float64))          # inside the window: untouched
    old = Veff[:n - R].reshape(n - R, 128 // Gv, Gv)
    orig = V[:n - R].astype(np.float64).reshape(n - R, 128 // Gv, Gv)
    mn, mx = orig.min(-1, keepdims=True), orig.max(-1, keepdims=True)
    step = (mx - mn) / (2 ** bits - 1)
    err = np.abs(old - orig)
    assert (err <= 0.5 * step * (1 + 2e-3) + 2e-3 * np.abs(orig) + 1e-6).all()
    assert (np.abs(old.min(-1, keepdims=True) - mn) <= 1e-3 * np.abs(mn) + 1e-6).all()  # the minimum is a level
    assert (err.reshape(n - R, -1).max(-1) > 0).all()                          # each of them was quantized
    # the two tokens on either side of the window's edge
    assert not np.array_equal(Veff[n - R - 1], V[n - R - 1].astype(np.float64))
    assert np.array_equal(Veff[n - R], V[n - R].astype(np.float64))


def test_values_between_the_two_quantized_lengths_are_fp16_levels():
    """Tokens whose Keys are still in full precision but whose Values are quantized are attended with
    the fp16 rounding of zero + code * step; below n_quant with the unrounded level."""
    G, R, n, bits, Gv = 32, 40, 32 * 3 + 40 + 20, 2, 32
    K, V = _rows(3, n)
    st = O.PerStepValueUnit(128, bits, G, Gv)
    st.advance_to(K, V, n, R)
    nq, nqv = st.n_quant, st.n_quant_v
    assert (nq, nqv) == (96, 116)
    Keff, Veff = st.effective_rows(K[nq:n], V[nq:n])
    assert np.array_equal(Keff[nq:], K[nq:n].astype(np.float64))                 # Keys of the ring: original
    codes = st.v_codes.astype(np.float64).reshape(nqv, 4, 32)
    exact = (st.v_zero.astype(np.float64)[..., None] + codes * st.v_step.astype(np.float64)[..., None]).reshape(nqv, 128)
    assert np.array_equal(Veff[:nq], exact[:nq])
    assert np.array_equal(Veff[nq:nqv], exact[nq:nqv].astype(np.float16).astype(np.float64))
    assert (Veff[nq:nqv] != exact[nq:nqv]).any()                                 # the rounding is really there


@pytest.mark.parametrize("n", [20, 128, 129, 200, 333])
def test_attention_is_library_attention_over_the_scheduled_rows(n):
    """decode_attention on a per-step unit = torch's scaled_dot_product_attention over explicitly
    assembled matrices (built here from the unit's codes, not by the oracle's own row assembly)."""
    G, R, bits, Gv = 32, 128, 2, 32
    K, V = _rows(4 + n, n)
    st = O.PerStepValueUnit(128, bits, G, Gv)
    for m in range(1, n + 1):                                                    # token by token, as in decoding
        st.advance_to(K, V, m, R)
    nq, nqv = st.n_quant, st.n_quant_v
    Kd = torch.from_numpy(K.astype(np.float64))
    Vd = torch.from_numpy(V.astype(np.float64))
    for t in range(nqv):
        lv = torch.zeros(128, dtype=torch.float64)
        for c in range(128):
            lv[c] = float(st.v_zero[t, c // Gv]) + float(st.v_codes[t, c]) * float(st.v_step[t, c // Gv])
        Vd[t] = lv if t < nq else lv.to(torch.float16).to(torch.float64)
    for t in range(nq):
        for c in range(128):
            Kd[t, c] = float(st.k_zero[t // G, c]) + float(st.k_codes[t, c]) * float(st.k_step[t // G, c])
    rng = np.random.default_rng(9)
    q = rng.standard_normal((2, 128)).astype(np.float16)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.astype(np.float64))[None], Kd[None], Vd[None])[0].numpy()
    got, got16 = O.decode_attention(q, st, K[nq:n], V[nq:n])
    assert np.abs(got - want).max() < 1e-12
    assert got16.dtype == np.float16


def test_everything_inside_the_window_is_plain_attention():
    n, R = 100, 128
    K, V = _rows(7, n)
    st = O.PerStepValueUnit(128, 2, 32, 32)
    st.advance_to(K, V, n, R)
    assert st.n_quant == 0 and st.n_quant_v == 0
    q = np.random.default_rng(1).standard_normal((1, 128)).astype(np.float16)
    got, _ = O.decode_attention(q, st, K, V)
    want = O.softmax_attention(q[0], K.astype(np.float64), V.astype(np.float64))
    assert np.array_equal(got[0], want)


def test_keys_cannot_close_before_their_values():
    st = O.PerStepValueUnit(128, 2, 32, 32)
    K, V = _rows(8, 64)
    with pytest.raises(AssertionError):
        st.append_key_group(K[:32])
    with pytest.raises(TypeError):
        st.append_group(K[:32], V[:32])
