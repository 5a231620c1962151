"""Pins for the oracle's decode attention (Eq. 1 over the three cache kinds) and for
its packer.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import kvq_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def build(n, N=4, A=32, G=32, R=32, bits=2, Gv=32, seed=0, frac=0.05):
    g = rng(seed)
    K = g.standard_normal((n, 128))
    K[:, [7, 50, 90, 120]] *= 20
    K[g.random(n) < frac] *= 0.05
    K = K.astype(np.float16)
    V = g.standard_normal((n, 128)).astype(np.float16)
    st = O.UnitState(128, bits, G, Gv, N, A)
    nq = G * ((n - R) // G) if n >= R + G else 0
    for i in range(nq // G):
        st.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
    return st, K, V, nq


def test_unquantized_equals_bruteforce_and_library():
    g = rng(1)
    n, hd = 40, 128
    K = g.standard_normal((n, hd)).astype(np.float16)
    V = g.standard_normal((n, hd)).astype(np.float16)
    Q = g.standard_normal((3, hd)).astype(np.float16)
    st = O.UnitState(hd, 2, 32, 32, 4, 32)           # shorter than R+G: nothing quantized
    out, out16 = O.decode_attention(Q, st, K, V)
    # brute force with python floats
    for j in range(3):
        logits = [sum(float(Q[j, c]) * float(K[t, c]) for c in range(hd)) / math.sqrt(hd) for t in range(n)]
        m = max(logits)
        w = [math.exp(l - m) for l in logits]
        z = sum(w)
        for c in (0, 63, 127):
            want = sum(w[t] * float(V[t, c]) for t in range(n)) / z
            assert abs(out[j, c] - want) < 1e-12
    # library routine
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q.astype(np.float32))[None, :, None, :],
        torch.from_numpy(K.astype(np.float32))[None, None].expand(1, 3, n, hd),
        torch.from_numpy(V.astype(np.float32))[None, None].expand(1, 3, n, hd))
    assert np.abs(ref[0, :, 0].numpy() - out).max() < 1e-5
    assert np.abs(out16.astype(np.float64) - out).max() <= np.abs(out).max() * 2.0 ** -11


def test_general_case_equals_materialised_cache():
    st, K, V, nq = build(300, N=4, R=32)
    assert nq == 256 and len(st.pool) == 4 and len(st.aux) > 0
    Q = rng(2).standard_normal((4, 128)).astype(np.float16)
    out, _ = O.decode_attention(Q, st, K[nq:], V[nq:])
    # second, structurally different path: dequantize element by element from the codes
    Kh = np.zeros((300, 128)); Vh = np.zeros((300, 128))
    for t in range(nq):
        gk = t // st.G
        for c in range(128):
            Kh[t, c] = float(st.k_zero[gk, c]) + int(st.k_codes[t, c]) * float(st.k_step[gk, c])
            Vh[t, c] = float(st.v_zero[t, c // st.Gv]) + int(st.v_codes[t, c]) * float(st.v_step[t, c // st.Gv])
    for m in st.pool + st.aux:
        Kh[m["idx"]] = K[m["idx"]]; Vh[m["idx"]] = V[m["idx"]]
    Kh[nq:] = K[nq:]; Vh[nq:] = V[nq:]
    logits = Kh @ Q.astype(np.float64).T / math.sqrt(128)
    p = np.exp(logits - logits.max(0)); p /= p.sum(0)
    assert np.abs(p.T @ Vh - out).max() < 1e-12
    # every token exactly once: weights over n tokens sum to one -> constant V gives that constant
    st2, K2, V2, nq2 = build(300, N=4, R=32)
    const = rng(3).standard_normal(128).astype(np.float16)
    for m in st2.pool + st2.aux:
        m["v"] = const.copy()
    st2.v_codes[:] = 0; st2.v_step[:] = 0
    st2.v_zero[:] = const.reshape(4, 32)[:, 0]         # dequantized V row = its group's zero
    cz = np.repeat(const.reshape(4, 32)[:, 0], 32)
    for m in st2.pool + st2.aux:
        m["v"] = cz.copy()
    out2, _ = O.decode_attention(Q, st2, K2[nq2:], np.tile(cz, (300 - nq2, 1)))
    assert np.abs(out2 - cz.astype(np.float64)).max() < 1e-12


def test_invariances():
    st, K, V, nq = build(200, N=4, R=32)
    g = rng(4)
    Q = g.standard_normal((2, 128)).astype(np.float16)
    kr, vr = K[nq:], V[nq:]
    out, _ = O.decode_attention(Q, st, kr, vr)
    # permuting residual tokens leaves the output unchanged
    perm = g.permutation(len(kr))
    out_p, _ = O.decode_attention(Q, st, kr[perm], vr[perm])
    assert np.abs(out_p - out).max() < 1e-12
    # pool order is irrelevant
    st.pool = st.pool[::-1]
    out_r, _ = O.decode_attention(Q, st, kr, vr)
    assert np.abs(out_r - out).max() < 1e-12
    # GQA: head j uses the shared kv head, same as running it alone
    for j in range(2):
        o1, _ = O.decode_attention(Q[j:j + 1], st, kr, vr)
        assert np.array_equal(o1[0], out[j])
    # masked placeholder codes do not matter
    st.k_codes[st.masked] = 3 - st.k_codes[st.masked]
    out_m, _ = O.decode_attention(Q, st, kr, vr)
    assert np.array_equal(out_m, out)


def test_softmax_shift_invariance_and_scale():
    g = rng(5)
    K = g.standard_normal((50, 128)); V = g.standard_normal((50, 128))
    q = g.standard_normal(128).astype(np.float16)
    o = O.softmax_attention(q, K, V)
    # adding a multiple of q/|q|^2 * c to every key shifts every logit by the same constant
    shift = 5.0 * q.astype(np.float64) / (q.astype(np.float64) @ q.astype(np.float64))
    assert np.abs(O.softmax_attention(q, K + shift, V) - o).max() < 1e-9
    # scale is 1/sqrt(d_k): two keys with q.k differing by sqrt(d) ln 3 get weights 3:1
    qq = np.zeros(128, np.float16); qq[0] = 1
    KK = np.zeros((2, 128)); KK[0, 0] = math.sqrt(128) * math.log(3)
    VV = np.zeros((2, 128)); VV[0, 0] = 1; VV[1, 1] = 1
    o2 = O.softmax_attention(qq, KK, VV)
    assert abs(o2[0] - 0.75) < 1e-12 and abs(o2[1] - 0.25) < 1e-12


def test_packer_against_hand_computed_positions_and_bijection():
    rows = []
    with open(os.path.join(HERE, "golden", "packed_layout_positions.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                kind, bits, t, c, byte, start = line.split()
                rows.append((kind, int(bits), int(t), int(c), int(byte), int(start)))
    assert len(rows) >= 20
    for kind, bits, t, c, byte, start in rows:
        for code in ((1 << bits) - 1, 1):               # all bits of the code, then its lowest bit alone
            codes = np.zeros((32, 128), np.uint8)
            codes[t, c] = code
            packed = (O.pack_k_block if kind == "K" else O.pack_v_block)(codes, bits)
            want = np.zeros(128 * bits, np.uint32)
            for i in range(bits):
                want[byte // 4] |= np.uint32(((code >> i) & 1) << ((start + i) % 32))
            assert np.array_equal(packed.view("<u4"), want), (kind, bits, t, c)
    # bijection: each (t, c) owns its own bits; all-ones fills every bit
    for bits in (2, 4):
        for fn in (O.pack_k_block, O.pack_v_block):
            full = fn(np.full((32, 128), (1 << bits) - 1, np.uint8), bits)
            assert np.all(full == 0xFF)
            g = rng(6)
            codes = g.integers(0, 1 << bits, (32, 128)).astype(np.uint8)
            packed = fn(codes, bits)
            acc = np.zeros_like(packed)
            for t in (0, 5, 31):
                for c in (0, 33, 127):
                    one = np.zeros((32, 128), np.uint8); one[t, c] = codes[t, c]
                    acc_one = fn(one, bits)
                    assert np.array_equal(acc_one & packed, acc_one)
    # meta planes and mask words
    km = O.pack_k_meta(np.arange(256, dtype=np.float16).reshape(2, 128), -np.arange(256, dtype=np.float16).reshape(2, 128))
    assert km.shape == (2, 2, 128) and km[1, 0, 5] == 133 and km[1, 1, 5] == -133
    st = np.arange(64 * 4, dtype=np.float16).reshape(64, 4)          # step of token t, group j = 4t + j
    vm = O.pack_v_meta(st, -st)
    assert vm.shape == (2, 256)
    assert vm[0, 0] == 0 and vm[0, 1] == 4 and vm[0, 2] == 1 and vm[0, 3] == 5      # pair 0: (t0,j0),(t1,j0),(t0,j1),(t1,j1)
    assert vm[0, (3 * 4 + 2) * 2 + 1] == 4 * 7 + 2                                    # token 7 = pair 3, e = 1, group 2
    assert vm[0, 128 + (3 * 4 + 2) * 2 + 1] == -(4 * 7 + 2)                           # zero of token 7, group 2
    assert vm[1, 128 + (15 * 4 + 3) * 2 + 1] == -(4 * 63 + 3)                         # token 63 = block 1, pair 15, e = 1
    mk = np.zeros(64, bool); mk[0] = mk[33] = mk[63] = True
    assert O.mask_words(mk).tolist() == [1, (1 << 1) | (1 << 31)]


# ---- the quantized segment as fp16 rows (inverse of Eq. 2) ----------------------------------------------

@pytest.mark.parametrize("bits,G,Gv", [(2, 32, 32), (4, 64, 128), (2, 128, 64)])
def test_fp16_rows_are_the_exact_reconstruction_rounded_once_more(bits, G, Gv):
    st, K, V, nq = build(G * 6 + 40, N=4, G=G, R=32, bits=bits, Gv=Gv, seed=3)
    kh, vh = st.rows_fp16()
    ke, ve = st.effective_rows(K[nq:], V[nq:])                 # exact reconstruction, fp64 (pinned above)
    for got, exact in ((kh, ke[:nq]), (vh, ve[:nq])):
        assert got.dtype == np.float16 and got.shape == (nq, 128)
        # fp16 spacing at the exact value; the fp32 sum adds at most 2^-24 relative before the final rounding
        ulp = np.maximum(np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64), 2.0 ** -24)
        assert np.all(np.abs(got.astype(np.float64) - exact) <= 0.5 * ulp + 2.0 ** -24 * np.abs(exact))
    # tokens in the pools come out as the input rows, bit for bit; the others within step/2 (+ rounding)
    held = sorted(m["idx"] for m in st.pool + st.aux)
    assert held and np.array_equal(kh[held].view(np.uint16), K[held].view(np.uint16))
    assert np.array_equal(vh[held].view(np.uint16), V[held].view(np.uint16))
    free = np.setdiff1d(np.arange(nq), held)
    kstep = np.repeat(st.k_step.astype(np.float64), G, axis=0)
    err = np.abs(kh[free].astype(np.float64) - K[free].astype(np.float64))
    assert np.all(err <= 0.5 * kstep[free] + np.spacing(np.abs(K[free])).astype(np.float64))


def test_fp16_rows_of_lattice_inputs_are_the_inputs():
    # inputs that sit on the quantization lattice: every group spans [-1, 0.5] in steps of 0.5 (2-bit:
    # zero -1, step 0.5), all exactly representable, so the reconstruction must return the inputs
    g = rng(9)
    G = 32
    levels = np.array([-1.0, -0.5, 0.0, 0.5])
    K = levels[g.integers(0, 4, (G * 3, 128))]
    V = levels[g.integers(0, 4, (G * 3, 128))]
    K[::G, :] = -1.0; K[1::G, :] = 0.5                         # every Key group (per channel) spans the range
    V[:, ::32] = -1.0; V[:, 1::32] = 0.5                       # every Value group (per token) too
    K, V = K.astype(np.float16), V.astype(np.float16)
    st = O.UnitState(128, 2, G, 32, 0, 0)
    for i in range(3):
        st.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
    assert np.all(st.k_step == np.float16(0.5)) and np.all(st.v_zero == np.float16(-1.0))
    kh, vh = st.rows_fp16()
    assert np.array_equal(kh, K) and np.array_equal(vh, V)
