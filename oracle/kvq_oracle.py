"""Plain CPU oracle for KV-cache quantization with outlier-token tracing.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct
definition that the HIP path is compared against.  It shares no code with the
HIP path and is imported only by tests, the smoke check and the benchmark's
cpu_baseline leg.  Everything is numpy; floating-point accumulation is fp64
unless the paper's method fixes a narrower type (the stored step/zero are fp16,
and the quantizer's threshold comparisons are done in fp32 so that any IEEE-754
device takes the same integer decision).

What follows the paper, by passage:

* `quantize_groups` / `dequantize`  - uniform quantization, Eq. 2 (Background,
  "Uniform Quantization"), applied per group ("Group Quantization").
* `quantize_kv_group`               - channel-wise Keys over a token group and
  token-wise Values (Method, "Quantization"; Appendix "Mathematical
  Formulation", last sentence).
* `l1_scores`                       - outlier score S_i = ||K_i||_1 (Appendix
  "Outlier Token Identification").
* `UnitState.trace`                 - competition mechanism, steps 1-4 of the
  Appendix "Competition Mechanism", plus the auxiliary pool and the stop rule of
  Method, "Quantization" (last two sentences).
* `mean_replace`                    - "replaced with the mean values of all
  tokens" (Method, "Quantization").
* `decode_attention`                - Eq. 1 over the three cache kinds (Method,
  "Decoding").
* `PerStepValueUnit`                - the other schedule the paper measures itself
  against (Experiments, "Details": the Keys are compressed every G steps, the
  Values at each step; Efficiency comparison: that per-step compression is what
  the method saves).  Same quantizer, no tracing.
* `rope_rotate`                     - NOT from the paper: the rotary position
  embedding (Su et al., "RoFormer", Eq. 34, in the half-split pairing of the
  LLaMA-family models the paper evaluates) that a serving stack applies to the
  query and the new Key before they reach the cache; here so that a decode launch
  that applies it itself can be checked.

Where the paper is silent or ambiguous a reading is taken; each is stated at the
function that implements it.

Pins: every function here is pinned by tests/test_oracle_*.py (closed forms,
brute force on tiny inputs, invariants, library routines).  The paper prints no
worked numerical example of the quantizer, the tracing or the attention, so no
golden value comes from the paper itself.
"""
from __future__ import annotations

import numpy as np

HEAD_DIM = 128          # packed layout below is defined for this head size
BLOCK_TOKENS = 32       # tokens per packed block


# --------------------------------------------------------------------------
# Uniform / group quantization (Eq. 2)
# --------------------------------------------------------------------------

def inv_levels_f32(bits: int) -> np.float32:
    """fp32 nearest to 1 / (2^bits - 1): the constant the step is multiplied by."""
    return np.float32(1.0 / float((1 << bits) - 1))


def quantize_groups(x: np.ndarray, bits: int):
    """Quantize each group x[..., :] (last axis = one group) to `bits` bits.

    Eq. 2 with "rounding function" read as round-to-nearest, ties up:
      step q  = (X_max - X_min) / (2^b - 1)   evaluated as fl32(fl32(max-min) * c_b)
                and then rounded (nearest-even) to fp16, the stored precision;
      zero    = X_min (already fp16);
      Q(x)    = number of half-integer thresholds (k + 1/2) * q, k = 0 .. 2^b-2,
                that fl32(x - X_min) reaches.  This is round-half-up of
                (x - X_min) / q clamped to [0, 2^b - 1], written without a
                division so the integer decision is the same on every IEEE
                machine.
    A group whose stored step is zero (constant group, or step underflow) gets
    all codes 0.  A minimum of zero is stored as +0: fp16 has two zeros that are
    the same number, and the stored pattern has to be one of them.

    Returns (codes uint8 [..., m], step fp16 [...], zero fp16 [...]).
    """
    assert x.dtype == np.float16
    levels = (1 << bits) - 1
    mn = x.min(axis=-1) + np.float16(0.0)                        # -0 + +0 = +0; every other value unchanged
    mx = x.max(axis=-1)
    d = mx.astype(np.float32) - mn.astype(np.float32)            # fl32
    s32 = (d * inv_levels_f32(bits)).astype(np.float32)          # fl32
    with np.errstate(over="ignore"):
        step = s32.astype(np.float16)                            # RNE to fp16
    sf = step.astype(np.float32)
    t = x.astype(np.float32) - mn.astype(np.float32)[..., None]  # fl32
    codes = np.zeros(x.shape, dtype=np.uint8)
    for k in range(levels):
        thr = (np.float32(k + 0.5) * sf).astype(np.float32)      # exact in fp32
        codes += (t >= thr[..., None]).astype(np.uint8)
    codes[np.broadcast_to((sf == 0)[..., None], codes.shape)] = 0
    return codes, step, mn.copy()


def dequantize(codes: np.ndarray, step: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """x_hat = X_min + Q * q, as exact real arithmetic carried in fp64."""
    return zero.astype(np.float64)[..., None] + codes.astype(np.float64) * step.astype(np.float64)[..., None]


# --------------------------------------------------------------------------
# Outlier score, mean replacement, K/V group quantization
# --------------------------------------------------------------------------

def l1_scores(k_rows: np.ndarray) -> np.ndarray:
    """S_t = sum_c |K[t, c]|, exact: fp16 magnitudes are multiples of 2^-24 below
    2^16, so an fp64 sum of up to 2^13 of them carries no rounding."""
    return np.abs(k_rows.astype(np.float64)).sum(axis=-1)


def group_mean_fp16(rows: np.ndarray) -> np.ndarray:
    """Per-channel mean over all tokens of the group: exact fp64 sum, divided by
    the token count, rounded to fp32 and then to fp16 (both nearest-even)."""
    s = rows.astype(np.float64).sum(axis=0)
    return (s / rows.shape[0]).astype(np.float32).astype(np.float16)


def mean_replace(k_group: np.ndarray, v_group: np.ndarray, selected: np.ndarray):
    """Working copies of the group with the selected tokens' K and V rows
    overwritten by the per-channel mean of the ORIGINAL rows of all tokens in
    the group (selected ones included)."""
    k = k_group.copy()
    v = v_group.copy()
    if selected.any():
        k[selected] = group_mean_fp16(k_group)
        v[selected] = group_mean_fp16(v_group)
    return k, v


def quantize_kv_group(k_group, v_group, selected, bits: int, group_v: int):
    """Quantize one group of G tokens: Keys channel-wise (one (step, zero) per
    channel over the G tokens), Values token-wise (one (step, zero) per token per
    `group_v` consecutive channels), after mean replacement of selected tokens.

    k_group, v_group: fp16 [G, hd]; selected: bool [G].
    Returns dict with k_codes [G, hd] u8, k_step/k_zero [hd] fp16,
    v_codes [G, hd] u8, v_step/v_zero [G, hd // group_v] fp16.
    """
    G, hd = k_group.shape
    k, v = mean_replace(k_group, v_group, np.asarray(selected, dtype=bool))
    kc, ks, kz = quantize_groups(np.ascontiguousarray(k.T), bits)        # [hd, G]
    vc, vs, vz = quantize_groups(v.reshape(G, hd // group_v, group_v), bits)
    return dict(k_codes=np.ascontiguousarray(kc.T), k_step=ks, k_zero=kz,
                v_codes=vc.reshape(G, hd), v_step=vs, v_zero=vz)


# --------------------------------------------------------------------------
# Outlier tracing: competition, auxiliary pool, stop rule
# --------------------------------------------------------------------------

class UnitState:
    """Cache state of one (layer, batch, kv-head) unit, in logical (unpacked) form."""

    def __init__(self, head_dim: int, bits: int, group_k: int, group_v: int,
                 outlier_budget: int, aux_capacity: int):
        self.hd, self.bits, self.G, self.Gv = head_dim, bits, group_k, group_v
        self.N, self.A = outlier_budget, aux_capacity
        self.pool = []      # list of dict(idx, score, k, v)
        self.aux = []
        self.frozen = False
        self.k_codes = np.zeros((0, head_dim), np.uint8)
        self.v_codes = np.zeros((0, head_dim), np.uint8)
        self.k_step = np.zeros((0, head_dim), np.float16)     # per group
        self.k_zero = np.zeros((0, head_dim), np.float16)
        self.v_step = np.zeros((0, head_dim // group_v), np.float16)   # per token
        self.v_zero = np.zeros((0, head_dim // group_v), np.float16)
        self.masked = np.zeros((0,), bool)   # token lives in pool or aux

    @property
    def n_quant(self):
        return self.k_codes.shape[0]

    def trace(self, k_group: np.ndarray, v_group: np.ndarray, group_index: int) -> np.ndarray:
        """One competition step for group `group_index` (tokens group_index*G ...).

        1. No budget, or tracing already stopped: nothing selected.
        2. Score the G tokens (L1); pool members keep their stored score.
        3. Order pool U group by (score, token index) ascending; the new pool is
           the first min(N, count) of them.
        4. Old members that fall out go to the auxiliary pool.  If they do not
           all fit, tracing stops for good and this step changes nothing.
        5. Otherwise the group tokens that entered the pool are `selected`; the
           pool stores bit-exact copies of their original K and V rows.
        """
        G = self.G
        selected = np.zeros(G, bool)
        if self.N == 0 or self.frozen:
            return selected
        scores = l1_scores(k_group)
        cand = [(m["score"], m["idx"], "old", i) for i, m in enumerate(self.pool)]
        cand += [(float(scores[t]), group_index * G + t, "new", t) for t in range(G)]
        cand.sort(key=lambda c: (c[0], c[1]))
        keep = cand[:min(self.N, len(cand))]
        kept_old = {c[3] for c in keep if c[2] == "old"}
        evicted = [m for i, m in enumerate(self.pool) if i not in kept_old]
        if len(self.aux) + len(evicted) > self.A:
            self.frozen = True
            return selected
        self.aux.extend(evicted)
        new_pool = [m for i, m in enumerate(self.pool) if i in kept_old]
        for c in keep:
            if c[2] == "new":
                t = c[3]
                selected[t] = True
                new_pool.append(dict(idx=c[1], score=c[0], k=k_group[t].copy(), v=v_group[t].copy()))
        self.pool = new_pool
        return selected

    def append_group(self, k_group: np.ndarray, v_group: np.ndarray, trace: bool = True):
        """Trace (optional), mean-replace, quantize and append one group."""
        gi = self.n_quant // self.G
        selected = self.trace(k_group, v_group, gi) if trace else np.zeros(self.G, bool)
        q = quantize_kv_group(k_group, v_group, selected, self.bits, self.Gv)
        self.k_codes = np.concatenate([self.k_codes, q["k_codes"]])
        self.v_codes = np.concatenate([self.v_codes, q["v_codes"]])
        self.k_step = np.concatenate([self.k_step, q["k_step"][None]])
        self.k_zero = np.concatenate([self.k_zero, q["k_zero"][None]])
        self.v_step = np.concatenate([self.v_step, q["v_step"]])
        self.v_zero = np.concatenate([self.v_zero, q["v_zero"]])
        self.masked = np.concatenate([self.masked, selected])
        return selected, q

    def effective_rows(self, k_res: np.ndarray, v_res: np.ndarray):
        """Per-token effective K and V rows (fp64) for all n tokens: residual tokens
        as stored, pool / auxiliary tokens as their stored full-precision rows,
        every other token as its dequantized row.  Each token appears once."""
        G = self.G
        nq = self.n_quant
        kh = dequantize(self.k_codes.reshape(-1, G, self.hd).transpose(0, 2, 1),
                        self.k_step, self.k_zero).transpose(0, 2, 1).reshape(nq, self.hd)
        vh = dequantize(self.v_codes.reshape(nq, self.hd // self.Gv, self.Gv),
                        self.v_step, self.v_zero).reshape(nq, self.hd)
        for m in self.pool + self.aux:
            kh[m["idx"]] = m["k"].astype(np.float64)
            vh[m["idx"]] = m["v"].astype(np.float64)
        return (np.concatenate([kh, k_res.astype(np.float64)]),
                np.concatenate([vh, v_res.astype(np.float64)]))


    def rows_fp16(self):
        """The quantized segment as fp16 rows, as a consumer that wants the cache as a matrix
        gets it: x_hat = X_min + Q * q (the inverse of Eq. 2) evaluated in fp32 - the product of a
        code and an fp16 step is exact there, the sum rounds once - and rounded to nearest fp16;
        pool / auxiliary tokens as their stored rows.  Returns (K, V), fp16 [n_quant, hd]."""
        G, nq = self.G, self.n_quant
        f32 = np.float32
        kc = self.k_codes.reshape(-1, G, self.hd).astype(f32)
        kh = (self.k_zero.astype(f32)[:, None, :] + kc * self.k_step.astype(f32)[:, None, :]).reshape(nq, self.hd)
        vc = self.v_codes.reshape(nq, self.hd // self.Gv, self.Gv).astype(f32)
        vh = (self.v_zero.astype(f32)[..., None] + vc * self.v_step.astype(f32)[..., None]).reshape(nq, self.hd)
        kh, vh = kh.astype(np.float16), vh.astype(np.float16)
        for m in self.pool + self.aux:
            kh[m["idx"]] = m["k"]
            vh[m["idx"]] = m["v"]
        return kh, vh


# --------------------------------------------------------------------------
# The per-step Value schedule (the comparison schedule of Experiments, "Details")
# --------------------------------------------------------------------------

def quantize_value_rows(v_rows: np.ndarray, bits: int, group_v: int):
    """Token-wise quantization of Value rows on their own (Eq. 2 per token and per
    `group_v` consecutive channels: a token's groups do not involve other tokens).

    v_rows: fp16 [n, hd].  Returns (codes u8 [n, hd], step fp16 [n, hd/group_v],
    zero fp16 [n, hd/group_v], v_hat fp16 [n, hd]) where v_hat = zero + code * step
    evaluated in fp32 (the product is exact, the sum rounds once) and rounded to
    nearest fp16: the row as a cache that holds dequantized rows in fp16 keeps it."""
    n, hd = v_rows.shape
    vc, vs, vz = quantize_groups(v_rows.reshape(n, hd // group_v, group_v), bits)
    f32 = np.float32
    v_hat = (vz.astype(f32)[..., None] + vc.astype(f32) * vs.astype(f32)[..., None]).reshape(n, hd)
    return vc.reshape(n, hd), vs, vz, v_hat.astype(np.float16)


class PerStepValueUnit(UnitState):
    """A unit whose Values are quantized at each step and whose Keys every G steps.

    Reading taken (the paper only names the schedule): with n tokens in the cache,
        Keys   : tokens below n_quant = G * floor((n - R) / G) are quantized in groups
                 of G, exactly as in `UnitState` (same ring rule);
        Values : tokens below n - R are quantized, token-wise, each at the step at
                 which it leaves the window of the R most recent tokens.
    No outlier tracing (the schedule belongs to the method without it): N = 0.
    A token's Value codes do not depend on when they are computed, so once its Key
    group closes the unit holds exactly what `UnitState` with N = 0 holds.  In
    between (Keys still in full precision, Values already quantized) the token is
    attended with its full-precision Key row and its dequantized Value row held in
    fp16 (`quantize_value_rows`: v_hat)."""

    def __init__(self, head_dim: int, bits: int, group_k: int, group_v: int):
        super().__init__(head_dim, bits, group_k, group_v, 0, 0)
        self.v_hat = np.zeros((0, head_dim), np.float16)    # dequantized rows, all quantized tokens

    @property
    def n_quant_v(self):
        return self.v_codes.shape[0]

    def quantize_values(self, v_rows: np.ndarray):
        """The next tokens (in order) leave the window: quantize their Value rows."""
        vc, vs, vz, v_hat = quantize_value_rows(v_rows, self.bits, self.Gv)
        self.v_codes = np.concatenate([self.v_codes, vc])
        self.v_step = np.concatenate([self.v_step, vs])
        self.v_zero = np.concatenate([self.v_zero, vz])
        self.v_hat = np.concatenate([self.v_hat, v_hat])

    def append_key_group(self, k_group: np.ndarray):
        """Close the next Key group: channel-wise quantization of its G rows.  Its
        tokens' Values must already be quantized."""
        assert self.n_quant + self.G <= self.n_quant_v, "Values of the group are quantized before its Keys"
        kc, ks, kz = quantize_groups(np.ascontiguousarray(k_group.T), self.bits)
        self.k_codes = np.concatenate([self.k_codes, np.ascontiguousarray(kc.T)])
        self.k_step = np.concatenate([self.k_step, ks[None]])
        self.k_zero = np.concatenate([self.k_zero, kz[None]])
        self.masked = np.concatenate([self.masked, np.zeros(self.G, bool)])

    def append_group(self, k_group, v_group, trace: bool = True):
        raise TypeError("per-step schedule: use quantize_values and append_key_group")

    def advance_to(self, K: np.ndarray, V: np.ndarray, n: int, residual: int):
        """Bring the unit to the state it has with tokens 0 .. n-1 in the cache
        (K, V: fp16 [>= n, hd], the unit's rows from token 0 on)."""
        nv = max(0, n - residual)
        if nv > self.n_quant_v:
            self.quantize_values(V[self.n_quant_v:nv])
        nk = self.G * ((n - residual) // self.G) if n >= residual + self.G else 0
        while self.n_quant < nk:
            self.append_key_group(K[self.n_quant:self.n_quant + self.G])

    def effective_rows(self, k_res: np.ndarray, v_res: np.ndarray):
        """k_res, v_res: the original rows of tokens n_quant .. n-1.  Tokens below
        n_quant: dequantized Keys and Values (exact, as in `UnitState`); tokens
        n_quant .. n_quant_v - 1: original Key row, v_hat as Value row; the rest:
        original rows."""
        G, nq, nqv = self.G, self.n_quant, self.n_quant_v
        kh = dequantize(self.k_codes.reshape(-1, G, self.hd).transpose(0, 2, 1),
                        self.k_step, self.k_zero).transpose(0, 2, 1).reshape(nq, self.hd)
        vh = dequantize(self.v_codes[:nq].reshape(nq, self.hd // self.Gv, self.Gv),
                        self.v_step[:nq], self.v_zero[:nq]).reshape(nq, self.hd)
        v_tail = v_res.astype(np.float64).copy()
        v_tail[:nqv - nq] = self.v_hat[nq:nqv].astype(np.float64)
        return np.concatenate([kh, k_res.astype(np.float64)]), np.concatenate([vh, v_tail])

    def rows_fp16(self):
        raise TypeError("not defined for the per-step schedule")


# --------------------------------------------------------------------------
# Decode attention (Eq. 1)
# --------------------------------------------------------------------------

def softmax_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """ATT = softmax(q K^T / sqrt(d_k)) V for one query row, fp64, max-subtracted."""
    logits = K @ q.astype(np.float64) / np.sqrt(np.float64(q.shape[-1]))
    p = np.exp(logits - logits.max())
    p /= p.sum()
    return p @ V


def decode_attention(q_heads: np.ndarray, state: UnitState, k_res: np.ndarray, v_res: np.ndarray):
    """Outputs for the g query heads that share this unit's kv head.

    q_heads: fp16 [g, hd].  Returns (fp64 [g, hd], fp16 [g, hd]); the fp16 one is
    the fp64 result rounded through fp32 (nearest-even twice)."""
    K, V = state.effective_rows(k_res, v_res)
    out = np.stack([softmax_attention(q, K, V) for q in q_heads])
    return out, out.astype(np.float32).astype(np.float16)


# --------------------------------------------------------------------------
# Rotary position embedding (not part of the paper's method; see the header)
# --------------------------------------------------------------------------

def rope_rotate(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate rows x[..., hd] (fp16) by the angles of one position.

    Channel i < hd/2 is paired with channel i + hd/2; the pair is the point
    (x_i, x_{i+hd/2}) of a plane, turned counter-clockwise by the angle whose
    cosine and sine are cos[i], sin[i] (fp32, the caller's table: frequencies,
    base and scaling are the caller's):
        y_i        = x_i cos_i - x_{i+hd/2} sin_i
        y_{i+hd/2} = x_{i+hd/2} cos_i + x_i sin_i
    Precision (a reading: the arithmetic decides stored fp16 Key rows, so it is
    fixed): each product and the sum are rounded to fp32 separately (no fused
    multiply-add), the result once more to fp16, nearest-even."""
    x = np.asarray(x)
    assert x.dtype == np.float16
    hd = x.shape[-1]
    c = np.asarray(cos, dtype=np.float32).reshape(hd // 2)
    s = np.asarray(sin, dtype=np.float32).reshape(hd // 2)
    a = x[..., : hd // 2].astype(np.float32)
    b = x[..., hd // 2:].astype(np.float32)
    ya = (a * c).astype(np.float32) - (b * s).astype(np.float32)
    yb = (b * c).astype(np.float32) + (a * s).astype(np.float32)
    with np.errstate(over="ignore"):               # beyond the fp16 range: infinity, as IEEE-754 rounds it
        return np.concatenate([ya.astype(np.float32), yb.astype(np.float32)], axis=-1).astype(np.float16)


# --------------------------------------------------------------------------
# Packed layout (written from the layout description, not from kernel code)
# --------------------------------------------------------------------------
# A block is 32 tokens x 128 channels of b-bit codes = 512*b bytes, seen as 64
# "lanes" of 8 "fields" of 8 codes.  Code x = 2*v + e (v in 0..3, e in 0..1) of a
# field occupies, inside a little-endian u32 word, the b bits that start at bit
#     b=2:  (16*e + 2*(v + 1) + 8*(f & 1)) mod 32           of word (f >> 1) of the lane's 4 words
#     b=4:  (16*e + 2 + 4*(v & 1) + 8*(v >> 1)) mod 32      of word (f & 3) of half (f >> 2)
# and continue, past bit 31, at bit 0 of the same word (the code is rotated into place);
# the lane's words live at byte  half*1024 + lane*16 + 4*word.
# K block: token t = 16*th + m, channel c = 32*cb + 8*r + x -> lane 16*r + m, field 4*th + cb.
# V block: channel c = 16*ct + n, token t = 8*r + x        -> lane 16*r + n, field ct.
# Meta (fp16): Key group = step[128] then zero[128]; Value block = step[16 pairs][NV][2] then
# zero[16 pairs][NV][2].

def _pack_fields(fields: np.ndarray, bits: int) -> np.ndarray:
    """fields: u8 [64 lanes, 8 fields, 8 codes] -> packed block bytes (u8 [512*bits])."""
    words = np.zeros((2 if bits == 4 else 1, 64, 4), dtype=np.uint32)
    for lane in range(64):
        for f in range(8):
            for x in range(8):
                v, e = x >> 1, x & 1
                code = int(fields[lane, f, x])
                if bits == 2:
                    start, half, word = (16 * e + 2 * (v + 1) + 8 * (f & 1)) % 32, 0, f >> 1
                else:
                    start, half, word = (16 * e + 2 + 4 * (v & 1) + 8 * (v >> 1)) % 32, f >> 2, f & 3
                placed = code << start                      # bits pushed past bit 31 re-enter at bit 0
                words[half, lane, word] |= np.uint32((placed & 0xFFFFFFFF) | (placed >> 32))
    return words.astype("<u4").view(np.uint8).reshape(-1)


def pack_k_block(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes: u8 [32 tokens, 128 channels] -> packed bytes."""
    assert codes.shape == (BLOCK_TOKENS, HEAD_DIM)
    fields = np.zeros((64, 8, 8), np.uint8)
    for t in range(32):
        th, m = divmod(t, 16)
        for c in range(128):
            cb, rem = divmod(c, 32)
            r, x = divmod(rem, 8)
            fields[16 * r + m, 4 * th + cb, x] = codes[t, c]
    return _pack_fields(fields, bits)


def pack_v_block(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes: u8 [32 tokens, 128 channels] -> packed bytes."""
    assert codes.shape == (BLOCK_TOKENS, HEAD_DIM)
    fields = np.zeros((64, 8, 8), np.uint8)
    for t in range(32):
        r, x = divmod(t, 8)
        for c in range(128):
            ct, n = divmod(c, 16)
            fields[16 * r + n, ct, x] = codes[t, c]
    return _pack_fields(fields, bits)


def pack_k_meta(step: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """Key meta of the groups of one unit: fp16 [groups, 2, 128] = steps, then zeros."""
    return np.stack([step, zero], axis=1).astype(np.float16)


def pack_v_meta(step: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """Value meta of one unit, per 32-token block: fp16 step[16 pairs][NV][2] (token 2p+e,
    value group j at (p*NV + j)*2 + e) followed by fp16 zero[16 pairs][NV][2], same indexing.
    step, zero: fp16 [n tokens, NV]; returns fp16 [n/32, 64*NV]."""
    n, nv = step.shape
    out = np.zeros((n // 32, 64 * nv), np.float16)
    for blk in range(n // 32):
        for t in range(32):
            for j in range(nv):
                out[blk, ((t >> 1) * nv + j) * 2 + (t & 1)] = step[32 * blk + t, j]
                out[blk, 32 * nv + ((t >> 1) * nv + j) * 2 + (t & 1)] = zero[32 * blk + t, j]
    return out


def mask_words(masked: np.ndarray) -> np.ndarray:
    """bool [n tokens] (n multiple of 32) -> u32 per 32-token block, bit t%32."""
    m = masked.reshape(-1, 32).astype(np.uint64)
    return (m << np.arange(32, dtype=np.uint64)).sum(axis=1).astype(np.uint32)


def packed_unit(state: UnitState):
    """Packed image of one unit's quantized cache, as the HIP path must produce it (the tokens
    below n_quant: a per-step unit's further Value tokens are not part of it)."""
    nb = state.n_quant // 32
    kc = np.stack([pack_k_block(state.k_codes[32 * i:32 * i + 32], state.bits) for i in range(nb)]) \
        if nb else np.zeros((0, 512 * state.bits), np.uint8)
    vc = np.stack([pack_v_block(state.v_codes[32 * i:32 * i + 32], state.bits) for i in range(nb)]) \
        if nb else np.zeros((0, 512 * state.bits), np.uint8)
    return dict(k_codes=kc, v_codes=vc,
                k_meta=pack_k_meta(state.k_step, state.k_zero),
                v_meta=pack_v_meta(state.v_step[:state.n_quant], state.v_zero[:state.n_quant]),
                mask=mask_words(state.masked))
