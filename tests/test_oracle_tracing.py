"""Pins for the oracle's outlier tracing, auxiliary pool, stop rule and mean
replacement (Method "Quantization"; Appendix "Competition Mechanism").  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import kvq_oracle as O


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def make_state(N, A, G=32, hd=128, bits=2, Gv=32):
    return O.UnitState(hd, bits, G, Gv, N, A)


def stream(state, K, V):
    G = state.G
    sels = []
    for i in range(K.shape[0] // G):
        s, _ = state.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
        sels.append(s)
    return np.concatenate(sels)


def test_scores_two_exact_methods():
    g = rng(1)
    K = (g.standard_normal((64, 128)) * g.choice([1e-3, 1, 100], size=(64, 1))).astype(np.float16)
    s = O.l1_scores(K)
    # independent exact method: integers in units of 2^-24
    ints = [sum(int(Fraction(float(abs(x))) * (1 << 24)) for x in row) for row in K]
    assert [int(Fraction(float(v)) * (1 << 24)) for v in s] == ints
    assert np.all(s >= 0)
    # L1, not L2 / max: a row of ones scores hd
    assert O.l1_scores(np.ones((1, 128), np.float16))[0] == 128.0
    assert O.l1_scores(-2 * np.ones((1, 128), np.float16))[0] == 256.0


@pytest.mark.parametrize("N,G", [(4, 32), (8, 32), (3, 128), (32, 32)])
def test_streaming_topn_equals_global_topn(N, G):
    g = rng(2)
    n = 8 * G
    K = g.standard_normal((n, 128)).astype(np.float16)
    K[g.random(n) < 0.05] *= np.float16(0.05)
    V = g.standard_normal((n, 128)).astype(np.float16)
    st = make_state(N, A=10 ** 6, G=G)        # aux never fills
    scores = np.abs(K.astype(np.float64)).sum(-1)
    ever = set()
    for i in range(n // G):
        st.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
        seen = (i + 1) * G
        order = sorted(range(seen), key=lambda t: (scores[t], t))
        want = set(order[:min(N, seen)])
        got = {m["idx"] for m in st.pool}
        assert got == want                                    # smaller score = more outlier
        ever |= got
        assert {m["idx"] for m in st.aux} == ever - got      # aux = ever-in-pool minus pool
        assert len({m["idx"] for m in st.pool + st.aux}) == len(st.pool) + len(st.aux)
    # stored rows are bit-exact copies, stored score is the row's L1
    for m in st.pool + st.aux:
        assert np.array_equal(m["k"].view(np.uint16), K[m["idx"]].view(np.uint16))
        assert np.array_equal(m["v"].view(np.uint16), V[m["idx"]].view(np.uint16))
        assert m["score"] == scores[m["idx"]]
    assert np.array_equal(np.flatnonzero(st.masked), sorted(m["idx"] for m in st.pool + st.aux))


def test_tie_break_by_token_index():
    K = np.ones((64, 128), np.float16)           # all scores equal
    V = np.zeros((64, 128), np.float16)
    st = make_state(4, 32)
    stream(st, K, V)
    assert sorted(m["idx"] for m in st.pool) == [0, 1, 2, 3]
    assert st.aux == []


def test_budget_zero_is_plain_group_quantization():
    g = rng(3)
    K = g.standard_normal((64, 128)).astype(np.float16)
    V = g.standard_normal((64, 128)).astype(np.float16)
    st = make_state(0, 32)
    sel = stream(st, K, V)
    assert not sel.any() and st.pool == [] and st.aux == [] and not st.frozen
    plain = O.quantize_kv_group(K[:32], V[:32], np.zeros(32, bool), 2, 32)
    assert np.array_equal(st.k_codes[:32], plain["k_codes"])
    assert np.array_equal(st.v_codes[:32], plain["v_codes"])


@pytest.mark.parametrize("A", [1, 3])
def test_freeze_exactly_when_aux_would_overflow(A):
    # descending norms: each group evicts the whole pool (N tokens)
    N, G = 2, 32
    groups = A + 3
    K = np.zeros((groups * G, 128), np.float16)
    for i in range(groups):
        K[i * G:(i + 1) * G] = np.float16(2.0 ** (groups - i))
        K[i * G:i * G + N] = np.float16(2.0 ** (groups - i) / 4)    # the N smallest of the group, smaller than all before
    V = np.zeros_like(K)
    st = make_state(N, A, G)
    log = []
    for i in range(groups):
        before = (sorted(m["idx"] for m in st.pool), sorted(m["idx"] for m in st.aux))
        sel, _ = st.append_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G])
        log.append((st.frozen, int(sel.sum())))
        if st.frozen:
            assert not sel.any()
            assert before == (sorted(m["idx"] for m in st.pool), sorted(m["idx"] for m in st.aux))
    # group 0 fills the pool (no eviction); group i>=1 evicts N=2; aux holds floor(A/2) evictions
    fits = A // N
    for i, (frozen, nsel) in enumerate(log):
        if i <= fits:
            assert not frozen and nsel == N
        else:
            assert frozen and nsel == 0
    assert len(st.aux) == fits * N <= A


def test_mean_replacement_pins():
    g = rng(4)
    G = 32
    K = g.standard_normal((G, 128)).astype(np.float16)
    K[:, 5] = (20 + 2 * g.standard_normal(G)).astype(np.float16)   # outlier channel with large mean
    K[9] *= np.float16(0.05)
    V = g.standard_normal((G, 128)).astype(np.float16)
    sel = np.zeros(G, bool)
    # nothing selected: identical to inputs
    k0, v0 = O.mean_replace(K, V, sel)
    assert np.array_equal(k0, K) and np.array_equal(v0, V)
    sel[9] = True
    k1, v1 = O.mean_replace(K, V, sel)
    assert np.array_equal(k1[~sel], K[~sel]) and np.array_equal(v1[~sel], V[~sel])
    # exact mean via rationals, then one rounding to fp32 and one to fp16
    for c in (0, 5, 77):
        fr = sum(Fraction(float(x)) for x in K[:, c]) / G
        want = np.float16(np.float32(float(fr)))     # float(Fraction) is correctly rounded to fp64; /G is exact
        assert k1[9, c] == want
        frv = sum(Fraction(float(x)) for x in V[:, c]) / G
        assert v1[9, c] == np.float16(np.float32(float(frv)))
    # placeholder lies inside the channel's original range, so the step cannot grow
    assert np.all(k1[9] >= K.min(0)) and np.all(k1[9] <= K.max(0))
    q_plain = O.quantize_kv_group(K, V, np.zeros(G, bool), 2, 32)
    q_ott = O.quantize_kv_group(K, V, sel, 2, 32)
    assert np.all(q_ott["k_step"].astype(np.float32) <= q_plain["k_step"].astype(np.float32))
    assert q_ott["k_step"][5] < q_plain["k_step"][5]     # the low-magnitude token widened channel 5


def test_retained_outliers_reduce_attention_error():
    # Qualitative claim of the preliminary study: keeping the smallest-norm tokens in full
    # precision lowers the attention-output loss; keeping the largest does not help as much.
    g = rng(5)
    n, hd, G = 256, 128, 32
    K = g.standard_normal((n, hd))
    ch = [3, 40, 77, 100]
    K[:, ch] = 20 * np.sign(g.standard_normal(4)) + 2 * g.standard_normal((n, 4))
    low = g.choice(n, 6, replace=False)
    K[low] *= 0.05
    K = K.astype(np.float16)
    V = g.standard_normal((n, hd)).astype(np.float16)
    Q = (0.1 * g.standard_normal((16, hd))).astype(np.float16)
    Q[:, ch] = (g.standard_normal((16, 4))).astype(np.float16)
    ref = np.stack([O.softmax_attention(q, K.astype(np.float64), V.astype(np.float64)) for q in Q])

    def loss(keep):
        st = make_state(0, 0)
        for i in range(n // G):
            sel = np.isin(np.arange(i * G, (i + 1) * G), keep)
            qz = O.quantize_kv_group(K[i * G:(i + 1) * G], V[i * G:(i + 1) * G], sel, 2, 32)
            st.k_codes = np.concatenate([st.k_codes, qz["k_codes"]]); st.v_codes = np.concatenate([st.v_codes, qz["v_codes"]])
            st.k_step = np.concatenate([st.k_step, qz["k_step"][None]]); st.k_zero = np.concatenate([st.k_zero, qz["k_zero"][None]])
            st.v_step = np.concatenate([st.v_step, qz["v_step"]]); st.v_zero = np.concatenate([st.v_zero, qz["v_zero"]])
        st.masked = np.isin(np.arange(n), keep)
        st.pool = [dict(idx=int(t), score=0.0, k=K[t], v=V[t]) for t in keep]
        out, _ = O.decode_attention(Q, st, np.zeros((0, hd), np.float16), np.zeros((0, hd), np.float16))
        return np.abs(out - ref).mean()

    norms = np.abs(K.astype(np.float64)).sum(-1)
    order = np.argsort(norms)
    l_none, l_small, l_large = loss([]), loss(order[:6]), loss(order[-6:])
    assert l_small < l_none
    assert l_small < l_large
