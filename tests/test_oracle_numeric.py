"""Pins for the numerical part of the CPU oracle: each check compares an oracle function with
something other than itself -- exact rational arithmetic, a closed form, an invariant, a
hand-worked example or brute force -- chosen so a dropped term, wrong index or transposed
operand fails at least one of them."""
import itertools
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import moe_oracle as O
from oracle import c_ffn


def frac16(v) -> Fraction:
    return Fraction(float(np.float16(v)))


# ------------------------------------------------------------------ top-k / softmax / routing

def full_sort_top(z, k):
    order = sorted(range(len(z)), key=lambda e: (-z[e], e))  # python's sort is stable and total here
    return order[:k]


def test_top_k_equals_full_sort_random():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(2, 12))
        z = rng.normal(size=n)
        k = int(rng.integers(1, n + 1))
        assert O.top_k(list(z), k) == full_sort_top(list(z), k)


def test_top_k_ties_and_adversarial():
    assert O.top_k([1.0] * 8, 2) == [0, 1]                      # all equal: lowest indices
    assert O.top_k([0.0, 3.0, 3.0, 1.0], 2) == [1, 2]           # tie for first
    assert O.top_k([5.0, 1.0, 2.0, 2.0], 2) == [0, 2]           # tie for second: lower index
    assert O.top_k([-1.0, -2.0, -0.0, 0.0], 2) == [2, 3]        # -0.0 == 0.0 is a tie
    assert O.top_k([0.5, 2.0, 1.0], 4) == [1, 2, 0]             # more asked for than there are: all, in order
    assert O.prefetch_guess(np.array([0.2, 0.7, 0.1]), 4) == [1, 0, 2]
    for vals in itertools.product([0.0, 1.0, 2.0], repeat=5):   # exhaustive small alphabet
        for k in (1, 2, 3):
            assert O.top_k(list(vals), k) == full_sort_top(list(vals), k)


def test_softmax_and_combine_weights_closed_form():
    rng = np.random.default_rng(1)
    for _ in range(200):
        E, H = 8, 64
        wg = rng.normal(size=(E, H)).astype(np.float32)
        h = rng.normal(size=H).astype(np.float16)
        idx, w, z = O.route(wg, h, 2)
        p = O.softmax(z)
        assert abs(p.sum() - 1.0) < 1e-12 and (p > 0).all()
        assert abs(w.sum() - 1.0) < 1e-12
        assert w[0] >= w[1]
        # renormalised top-2 softmax == logistic of the logit gap
        assert abs(w[0] - 1.0 / (1.0 + math.exp(z[idx[1]] - z[idx[0]]))) < 1e-12
        assert idx == full_sort_top(list(z), 2)
    # softmax is shift invariant and monotone
    z = np.array([0.3, -1.2, 2.0, 0.0])
    assert np.allclose(O.softmax(z), O.softmax(z + 100.0), atol=1e-15)
    assert list(np.argsort(-O.softmax(z))) == list(np.argsort(-z))


def test_gate_logits_against_exact_rational_sum():
    rng = np.random.default_rng(2)
    E, H = 5, 48   # non-square so a transposed operand cannot pass
    wg = (rng.normal(size=(E, H)) * 0.02).astype(np.float32)
    h = rng.normal(size=H).astype(np.float16)
    z = O.gate_logits(wg, h)
    for e in range(E):
        exact = sum(Fraction(float(wg[e, i])) * Fraction(float(h[i])) for i in range(H))
        assert abs(Fraction(float(z[e])) - exact) <= abs(exact) * Fraction(1, 10**13) + Fraction(1, 10**18)


# ------------------------------------------------------------------ quantizer and dequantizer

def test_quantizer_hand_worked_examples(golden_dir):
    with open(os.path.join(golden_dir, "quantizer_worked_example.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        w = np.array(c["w"], dtype=np.float32)
        q, s, z = O.quantize_minmax(w, c["bits"], c["group"])
        assert q.tolist() == c["codes"]
        assert s.astype(np.float64).tolist() == c["scale"]
        assert z.astype(np.float64).tolist() == c["zero"]
        assert O.dequantize(q, s, z, c["group"]).tolist() == c["dequant"]


@pytest.mark.parametrize("bits,group", [(4, 64), (3, 64), (2, 16)])
def test_quantizer_range_extremes_and_roundtrip_bound(bits, group):
    rng = np.random.default_rng(3 + bits)
    w = (rng.normal(size=(24, 4 * group)) * 0.02).astype(np.float32)
    w[5, :group] = 0.0125                      # a constant group
    q, s, z = O.quantize_minmax(w, bits, group)
    qmax = (1 << bits) - 1
    assert q.dtype == np.uint8 and q.min() >= 0 and q.max() <= qmax
    assert s.shape == (24, 4) and z.shape == (24, 4) and s.dtype == np.float16
    wg = w.reshape(24, 4, group)
    qg = q.reshape(24, 4, group)
    lo, hi = wg.min(axis=2), wg.max(axis=2)
    nonconst = hi > lo
    # the group minimum takes code 0 and the maximum the top code
    assert (np.take_along_axis(qg, wg.argmin(axis=2)[..., None], 2)[..., 0][nonconst] == 0).all()
    assert (np.take_along_axis(qg, wg.argmax(axis=2)[..., None], 2)[..., 0][nonconst] == qmax).all()
    assert (qg[~nonconst] == 0).all() and (s[~nonconst] == 1).all()
    # |w - w^| <= s/2 (rounding) + qmax|s - s_exact| + s|z - z_exact| (metadata rounding, clipping)
    sd, zd = s.astype(np.float64), z.astype(np.float64)
    s_exact = np.where(nonconst, (hi.astype(np.float64) - lo) / qmax, 1.0)
    z_exact = -lo.astype(np.float64) / sd
    bound = sd / 2 + qmax * np.abs(sd - s_exact) + sd * np.abs(zd - z_exact) + 1e-7
    err = np.abs(O.dequantize(q, s, z, group).reshape(24, 4, group) - wg)
    assert (err <= bound[..., None]).all()
    # and the bound is not vacuous: typical error is a sizeable fraction of s/2
    assert err[nonconst].mean() > 0.2 * (sd[nonconst] / 2).mean()


def test_dequantize_against_exact_rational_definition():
    rng = np.random.default_rng(4)
    rows, cols, g = 3, 12, 4   # non-square, 3 groups per row with distinct metadata
    q = rng.integers(0, 16, size=(rows, cols)).astype(np.uint8)
    s = rng.uniform(0.001, 0.02, size=(rows, cols // g)).astype(np.float16)
    z = rng.uniform(0.0, 15.0, size=(rows, cols // g)).astype(np.float16)
    w = O.dequantize(q, s, z, g)
    for r in range(rows):
        for c in range(cols):
            exact = (Fraction(int(q[r, c])) - frac16(z[r, c // g])) * frac16(s[r, c // g])
            assert abs(Fraction(float(w[r, c])) - exact) <= abs(exact) * Fraction(1, 10**15)


def test_group_factorisation_identity():
    """sum_i (q_i - z) s h_i == s (sum_i q_i h_i - z sum_i h_i) per group: the algebra a fused kernel may use."""
    rng = np.random.default_rng(5)
    g = 64
    q = rng.integers(0, 16, size=(1, g)).astype(np.uint8)
    s = np.array([[0.0071]], dtype=np.float16)
    z = np.array([[7.43]], dtype=np.float16)
    h = rng.normal(size=g).astype(np.float16).astype(np.float64)
    direct = float(O.dequantize(q, s, z, g)[0] @ h)
    fact = float(s[0, 0]) * (float(q[0].astype(np.float64) @ h) - float(z[0, 0]) * h.sum())
    assert abs(direct - fact) < 1e-12 * max(1.0, abs(direct))


# ------------------------------------------------------------------ expert FFN

def rand_expert(rng, H, F, bits, g):
    out = []
    for shape in ((F, H), (F, H), (H, F)):
        q = rng.integers(0, 1 << bits, size=shape).astype(np.uint8)
        s = rng.uniform(0.002, 0.01, size=(shape[0], shape[1] // g)).astype(np.float16)
        z = rng.uniform(0.0, (1 << bits) - 1, size=(shape[0], shape[1] // g)).astype(np.float16)
        out.append((q, s, z))
    return out


def brute_ffn(h, expert, g):
    """Pure-python, exactly summed (math.fsum) evaluation of the definition."""
    H = len(h)
    hf = [float(x) for x in h]

    def mat(m, vec):
        q, s, z = m
        rows, cols = q.shape
        return [math.fsum((float(q[r, c]) - float(z[r, c // g])) * float(s[r, c // g]) * vec[c]
                          for c in range(cols)) for r in range(rows)]
    u = mat(expert[0], hf)
    v = mat(expert[1], hf)
    a = [ui / (1.0 + math.exp(-ui)) * vi for ui, vi in zip(u, v)]
    y = mat(expert[2], a)
    assert len(y) == H
    return np.array(y)


@pytest.mark.parametrize("bits,g", [(4, 4), (3, 4), (2, 2)])
def test_expert_ffn_against_brute_force(bits, g):
    rng = np.random.default_rng(6)
    H, F = 8, 12
    ex = rand_expert(rng, H, F, bits, g)
    h = rng.normal(size=H).astype(np.float16)
    ref = brute_ffn(h, ex, g)
    assert np.allclose(O.expert_ffn(h, ex, g), ref, rtol=1e-12, atol=1e-14)
    assert np.allclose(c_ffn.expert_ffn(h, ex, g), ref, rtol=1e-12, atol=1e-14)


def test_expert_ffn_textbook_special_case():
    """scale 1, zero 0, W1 = 2I, W3 = I, W2 = 3I  =>  y = 3 * silu(2h) * h elementwise.
    Swapping w1 and w3, or applying silu to the wrong branch, changes the result."""
    H = 8
    eye = np.eye(H, dtype=np.uint8)
    one = np.ones((H, 2), dtype=np.float16)
    zero = np.zeros((H, 2), dtype=np.float16)
    ex = [(2 * eye, one, zero), (eye, one, zero), (3 * eye, one, zero)]
    h = np.linspace(-2, 2, H).astype(np.float16)
    hd = h.astype(np.float64)
    want = 3.0 * (2 * hd / (1.0 + np.exp(-2 * hd))) * hd
    assert np.allclose(O.expert_ffn(h, ex, 4), want, rtol=1e-14)
    assert np.allclose(c_ffn.expert_ffn(h, ex, 4), want, rtol=1e-14)
    swapped = [ex[1], ex[0], ex[2]]
    assert not np.allclose(O.expert_ffn(h, swapped, 4), want, rtol=1e-6)


@pytest.mark.parametrize("bits,g,H,F", [(4, 64, 256, 512), (3, 64, 128, 320), (2, 16, 96, 160)])
def test_c_loops_equal_numpy_dense(bits, g, H, F):
    rng = np.random.default_rng(7)
    ex = rand_expert(rng, H, F, bits, g)
    for _ in range(3):
        h = rng.normal(size=H).astype(np.float16)
        a = O.expert_ffn(h, ex, g)
        b = c_ffn.expert_ffn(h, ex, g)
        assert np.abs(a - b).max() <= 1e-12 * np.abs(a).max()


# ------------------------------------------------------------------ second quantization level

def test_two_level_quantizer_hand_worked_examples(golden_dir):
    with open(os.path.join(golden_dir, "quantizer_two_level_worked_example.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        s16, z16 = np.array(c["scale"], dtype=np.float16), np.array(c["zero"], dtype=np.float16)
        qs, qz, meta, run = O.quantize_meta8(s16, z16, c["scale_group"])
        assert qs.tolist() == c["scale_codes"] and qz.tolist() == c["zero_codes"]
        assert meta.astype(np.float64).tolist() == c["meta"] and run == min(c["scale_group"], s16.shape[1])
        s, z = O.meta8_scale_zero(qs, qz, meta, run)
        assert s.tolist() == c["scale_decoded"] and z.tolist() == c["zero_decoded"]


def test_two_level_dequantize_against_exact_rational_definition():
    """weight = (q - zero) * scale with scale = (scale code - m1) * m0 and zero = (zero code - m3) * m2, the four
    m's shared by a run of consecutive groups of the row: exact rational arithmetic on non-square matrices with
    several runs per row, the last one whole or shorter, and distinct metadata everywhere (a transposed or
    mis-indexed run shows)."""
    for groups, run in ((6, 3), (7, 4), (5, 2)):
        check_two_level_exact(groups, run)


def check_two_level_exact(groups, run):
    rng = np.random.default_rng(14)
    rows, g, runs = 3, 4, -(-groups // run)
    q = rng.integers(0, 16, size=(rows, groups * g)).astype(np.uint8)
    qs = rng.integers(0, 256, size=(rows, groups)).astype(np.uint8)
    qz = rng.integers(0, 256, size=(rows, groups)).astype(np.uint8)
    meta = np.stack([rng.uniform(1e-5, 1e-4, (rows, runs)), rng.uniform(-40, 0, (rows, runs)),
                     rng.uniform(0.01, 0.06, (rows, runs)), rng.uniform(-5, 5, (rows, runs))], axis=2).astype(np.float16)
    w = O.dequantize_meta8(q, qs, qz, meta, run, g)
    for r in range(rows):
        for c in range(groups * g):
            j, k = c // g, c // g // run
            sc = (Fraction(int(qs[r, j])) - frac16(meta[r, k, 1])) * frac16(meta[r, k, 0])
            ze = (Fraction(int(qz[r, j])) - frac16(meta[r, k, 3])) * frac16(meta[r, k, 2])
            exact = (Fraction(int(q[r, c])) - ze) * sc
            assert abs(Fraction(float(w[r, c])) - exact) <= abs(exact) * Fraction(1, 10**14) + Fraction(1, 10**30)


def test_two_level_quantizer_codes_runs_and_roundtrip_bound():
    """Codes use the whole 8-bit range per run (run minimum -> 0, maximum -> 255), rows shorter than the scale
    group form one run, and a decoded scale is within half a step (plus the rounding of the run's fp16 pair)."""
    rng = np.random.default_rng(15)
    w = (rng.normal(size=(16, 8 * 64)) * 0.02).astype(np.float32)
    q, s16, z16 = O.quantize_minmax(w, 4, 64)                       # 8 groups per row
    for scale_group, runs in ((4, 2), (8, 1), (256, 1)):
        qs, qz, meta, r = O.quantize_meta8(s16, z16, scale_group)
        assert qs.dtype == np.uint8 and meta.shape == (16, runs, 4) and meta.dtype == np.float16
        assert r == 8 // runs
        for arr16, codes, j in ((s16, qs, 0), (z16, qz, 2)):
            v = arr16.astype(np.float64).reshape(16, runs, r)
            cg = codes.reshape(16, runs, r).astype(np.int64)
            lo, hi = v.min(axis=2), v.max(axis=2)
            step, zero = meta[:, :, j].astype(np.float64), meta[:, :, j + 1].astype(np.float64)
            # run minimum -> code 0; the maximum reaches the top code up to the rounding of the run's fp16 pair
            # (255 codes times a 2^-11 relative error of the step, plus the zero's own rounding)
            assert (np.take_along_axis(cg, v.argmin(axis=2)[..., None], 2)[..., 0] <= 1).all()
            assert (np.take_along_axis(cg, v.argmax(axis=2)[..., None], 2)[..., 0] >= 250).all()
            # |v - v^| <= step/2 + 255 |step - step_exact| + step |zero - zero_exact|, as for the first level
            step_exact = np.where(hi > lo, (hi - lo) / 255.0, 1.0)
            bound = step / 2 + 255 * np.abs(step - step_exact) + step * np.abs(zero - (-lo / step)) + 1e-9
            dec = (cg - zero[..., None]) * step[..., None]
            assert (np.abs(dec - v) <= bound[..., None]).all()
            assert np.abs(dec - v).mean() > 0.1 * (step / 2).mean()
        s, z = O.meta8_scale_zero(qs, qz, meta, r)
        assert np.array_equal(s.reshape(16, runs, r), (qs.reshape(16, runs, r) - meta[:, :, 1:2].astype(np.float64)) * meta[:, :, 0:1].astype(np.float64))
    # the weights the two-level form stands for stay close to the one-level ones
    qs, qz, meta, r = O.quantize_meta8(s16, z16, 256)
    w1, w2 = O.dequantize(q, s16, z16, 64), O.dequantize_meta8(q, qs, qz, meta, r, 64)
    assert np.abs(w1 - w2).max() < 0.02 * np.abs(w1).max()


def test_two_level_quantizer_short_last_run_equals_runs_quantized_one_by_one():
    """A row whose groups do not divide into whole runs (Sec. 4.2's 3-bit scheme: 224 groups of 64 along Mixtral's
    14336-wide rows, scale group 128) ends in a shorter run, quantized from its own minimum and maximum: the
    result equals quantizing every run of every row separately with the (pinned) first-level routine."""
    rng = np.random.default_rng(17)
    for bits, g, groups, scale_group in ((3, 64, 7, 4), (2, 16, 11, 4), (4, 64, 5, 2), (3, 64, 224, 128)):
        rows = 5 if groups < 100 else 2
        w = (rng.normal(size=(rows, groups * g)) * 0.02).astype(np.float32)
        q, s16, z16 = O.quantize_minmax(w, bits, g)
        qs, qz, meta, r = O.quantize_meta8(s16, z16, scale_group)
        runs = -(-groups // scale_group)
        assert r == scale_group and qs.shape == (rows, groups) and meta.shape == (rows, runs, 4)
        for j in range(runs):
            lo, hi = j * r, min(groups, (j + 1) * r)
            for arr16, codes, k in ((s16, qs, 0), (z16, qz, 2)):
                c1, s1, z1 = O.quantize_minmax(arr16[:, lo:hi].astype(np.float32), 8, hi - lo, zero_limit=O.META8_ZERO_LIMIT)
                assert np.array_equal(codes[:, lo:hi], c1)
                assert np.array_equal(meta[:, j, k].view(np.uint16), s1[:, 0].view(np.uint16))
                assert np.array_equal(meta[:, j, k + 1].view(np.uint16), z1[:, 0].view(np.uint16))
        s, z = O.meta8_scale_zero(qs, qz, meta, r)
        for gi in range(groups):
            m = meta[:, gi // r].astype(np.float64)
            assert np.array_equal(s[:, gi], (qs[:, gi] - m[:, 1]) * m[:, 0]) and np.array_equal(z[:, gi], (qz[:, gi] - m[:, 3]) * m[:, 2])


@pytest.mark.parametrize("bits,g,H,F,R", [(4, 64, 256, 512, 4), (3, 64, 320, 448, 4), (2, 16, 96, 160, 4)])
def test_two_level_c_loops_equal_numpy_dense(bits, g, H, F, R):
    rng = np.random.default_rng(16)
    ex = []
    for r, c in ((F, H), (F, H), (H, F)):
        w = (rng.normal(size=(r, c)) * 0.02).astype(np.float32)
        q, s16, z16 = O.quantize_minmax(w, bits, g)
        ex.append((q,) + O.quantize_meta8(s16, z16, R))
    for _ in range(3):
        h = rng.normal(size=H).astype(np.float16)
        a = O.expert_ffn(h, ex, g)
        dense = O.dequantize_meta8(*ex[2], g) @ (O.silu(O.dequantize_meta8(*ex[0], g) @ h.astype(np.float64))
                                                 * (O.dequantize_meta8(*ex[1], g) @ h.astype(np.float64)))
        assert np.abs(a - dense).max() <= 1e-13 * np.abs(dense).max()
        assert np.abs(a - c_ffn.expert_ffn(h, ex, g)).max() <= 1e-12 * np.abs(a).max()


def test_c_oracle_rejects_ragged_groups():
    rng = np.random.default_rng(8)
    ex = rand_expert(rng, 8, 12, 4, 4)
    with pytest.raises(ValueError):
        c_ffn.expert_ffn(np.zeros(8, np.float16), ex, 5)


# ------------------------------------------------------------------ RMSNorm and the block

def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(9)
    H, eps = 512, 1e-5
    x = (rng.normal(size=H) * 3).astype(np.float16)
    g = np.ones(H, dtype=np.float16)
    h = O.rmsnorm(x, g, eps)
    assert h.dtype == np.float16
    xs = [float(v) for v in x]
    ms = math.fsum(v * v for v in xs) / H
    e32 = float(np.float32(eps))
    want = np.array([v / math.sqrt(ms + e32) for v in xs]).astype(np.float16)
    assert (h == want).all()
    # gamma = 1: output rms = 1/sqrt(1 + eps/ms) up to fp16 rounding
    rms = math.sqrt(float((h.astype(np.float64) ** 2).mean()))
    assert abs(rms - 1.0 / math.sqrt(1.0 + e32 / ms)) < 1e-3
    # constant vector: h = c / sqrt(c^2 + eps)
    c = np.full(H, 0.5, dtype=np.float16)
    assert (O.rmsnorm(c, g, eps) == np.float16(0.5 / math.sqrt(0.25 + e32))).all()
    # eps matters when x is small: c = 2^-8 has c^2 = 1.5e-5, comparable to eps; and the zero vector stays zero
    small = np.full(H, 2.0 ** -8, dtype=np.float16)
    assert (O.rmsnorm(small, g, eps) == np.float16(2.0 ** -8 / math.sqrt(2.0 ** -16 + e32))).all()
    assert float(O.rmsnorm(small, g, eps)[0]) < 0.8
    assert (O.rmsnorm(np.zeros(H, np.float16), g, eps) == 0).all()
    # gain is applied per element, after the normalisation
    g2 = g.copy(); g2[7] = 2.0
    h2 = O.rmsnorm(x, g2, eps)
    assert h2[7] == np.float16(2.0 * xs[7] / math.sqrt(ms + e32)) and (np.delete(h2, 7) == np.delete(h, 7)).all()
    # batched input normalises each row on its own
    xb = np.stack([x, (x.astype(np.float32) * 0.25).astype(np.float16)])
    hb = O.rmsnorm(xb, g, eps)
    assert (hb[0] == h).all() and (hb[1] == O.rmsnorm(xb[1], g, eps)).all()


def test_moe_block_invariants():
    rng = np.random.default_rng(10)
    H, F, E, g = 32, 48, 6, 16
    experts = [rand_expert(rng, H, F, 4, g) for _ in range(E)]
    wg = rng.normal(size=(E, H)).astype(np.float32)
    x = rng.normal(size=H).astype(np.float16)
    r = O.moe_block(x, wg, experts, g, 2)
    # y is the weighted sum of the two selected experts and x_out the rounded residual
    want = sum(r.w[j] * brute_ffn(r.h, experts[e], g) for j, e in enumerate(r.idx))
    assert np.allclose(r.y, want, rtol=1e-11, atol=1e-13)
    assert (r.x_out == (x.astype(np.float64) + r.y).astype(np.float16)).all()
    assert (r.h == x).all()
    # identical experts: the weights sum to 1, so y is one expert's output whatever the routing
    same = [experts[0]] * E
    r2 = O.moe_block(x, wg, same, g, 2)
    assert np.allclose(r2.y, O.expert_ffn(x, experts[0], g), rtol=1e-12)
    # permuting the experts permutes the routing and leaves y unchanged
    perm = rng.permutation(E)
    r3 = O.moe_block(x, wg[perm], [experts[p] for p in perm], g, 2)
    assert [int(perm[i]) for i in r3.idx] == r.idx and np.allclose(r3.y, r.y, rtol=1e-12)
    # with the norm in front, the gate and the experts see h, the residual adds to x
    gam = np.ones(H, np.float16)
    r4 = O.moe_block(x, wg, experts, g, 2, gam, 1e-5)
    assert (r4.h == O.rmsnorm(x, gam, 1e-5)).all()
    r4b = O.moe_block(r4.h, wg, experts, g, 2)
    assert r4.idx == r4b.idx and np.allclose(r4.y, r4b.y, rtol=1e-12)
    assert (r4.x_out == (x.astype(np.float64) + r4.y).astype(np.float16)).all()


def test_paper_parameter_count(golden_dir):
    """Sec. 4.2 prints 45.1B expert parameters of 46.7B (96.6%): pins the Mixtral shapes used."""
    from workload import CONFIGS
    with open(os.path.join(golden_dir, "paper_constants.json")) as f:
        c = json.load(f)
    s = CONFIGS["mixtral_stack"]
    n = s.layers * s.n_experts * 3 * s.hidden * s.ffn
    assert n == 45_097_156_608
    assert round(n / 1e9, 1) == c["expert_params_billion"]["value"]
    assert round(100 * n / (c["total_params_billion"]["value"] * 1e9), 1) == c["expert_share_percent"]["value"]
    assert s.top_k == c["active_experts"]["value"] and s.cache_slots in c["cache_slots"]["value"]
    assert s.prefetch_m in c["prefetch_experts"]["value"]
