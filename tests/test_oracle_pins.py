"""Pins for the CPU oracle: each test checks it against something other than itself --
a closed form, a library routine, a numerical integral, a brute-force search, or a value the
paper prints (tests/golden/).  All CPU-only."""
import itertools
import math

import numpy as np
import pytest
import scipy.integrate
import scipy.linalg
import scipy.stats

from conftest import read_golden_rows
from oracle import polykv_oracle as O


# ------------------------------------------------------------------ FWHT ---
@pytest.mark.parametrize("d", [2, 8, 64, 128])
def test_fwht_equals_dense_sylvester_matrix(d):
    rng = np.random.default_rng(d)
    x = rng.standard_normal((5, d))
    H = scipy.linalg.hadamard(d).astype(np.float64)
    np.testing.assert_allclose(O.fwht(x), x @ H.T, rtol=0, atol=1e-11)
    # natural order: entry (i, j) is (-1)^popcount(i & j)
    i, j = 37 % d, 21 % d
    e = np.zeros(d); e[j] = 1.0
    assert O.fwht(e)[i] == (-1) ** bin(i & j).count("1")


@pytest.mark.parametrize("d", [64, 128])
def test_fwht_involution_parseval_special_vectors(d):
    rng = np.random.default_rng(7)
    xi = rng.integers(-50, 50, size=(3, d)).astype(np.float64)
    assert np.array_equal(O.fwht(O.fwht(xi)), d * xi)            # H.H = d.I, exact on integers
    x = rng.standard_normal((4, d))
    y = O.fwht(x) / math.sqrt(d)
    np.testing.assert_allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-13)
    e0 = np.zeros(d); e0[0] = 1.0
    assert np.array_equal(O.fwht(e0), np.ones(d))
    assert np.array_equal(O.fwht(np.ones(d)), d * e0)
    with pytest.raises(ValueError):
        O.fwht(np.zeros(48))


# -------------------------------------------------------------- codebook ---
def test_codebook_rounds_to_paper_values():
    printed = np.array([float(v) for v in read_golden_rows("paper_centroids.txt")[0]])
    c, _ = O.codebook()
    assert c.shape == (8,)
    np.testing.assert_array_equal(np.round(c, 3), printed)


def test_codebook_fixed_point_by_numerical_integration():
    c, t = O.codebook()
    assert np.all(np.diff(c) > 0)
    np.testing.assert_allclose(c, -c[::-1], atol=1e-15)           # odd symmetry
    np.testing.assert_allclose(t, 0.5 * (c[:-1] + c[1:]), atol=1e-15)
    assert abs(t[3]) < 1e-15
    pdf = scipy.stats.norm.pdf
    edges = [-np.inf, *t, np.inf]
    masses = []
    for k in range(8):
        num, _ = scipy.integrate.quad(lambda x: x * pdf(x), edges[k], edges[k + 1], epsabs=1e-13)
        den, _ = scipy.integrate.quad(pdf, edges[k], edges[k + 1], epsabs=1e-13)
        assert abs(num / den - c[k]) < 1e-9                        # centroid = conditional mean
        masses.append(den)
    assert abs(sum(masses) - 1.0) < 1e-10


def test_codebook_distortion_against_integral_and_paper_bound():
    c, t = O.codebook()
    pdf = scipy.stats.norm.pdf
    edges = [-np.inf, *t, np.inf]
    mse = sum(scipy.integrate.quad(lambda x, ck=c[k]: (x - ck) ** 2 * pdf(x),
                                   edges[k], edges[k + 1], epsabs=1e-13)[0] for k in range(8))
    assert abs(mse - O.lloyd_max_mse(c, t)) < 1e-10
    consts = {r[0]: float(r[1]) for r in read_golden_rows("paper_constants.txt")}
    assert round(mse, 2) == consts["distortion_b3"]                # "approximately 0.03"
    bound = O.turboquant_mse_bound(3)
    assert round(bound * 4 ** 3, 1) == consts["bound_factor"]      # sqrt(3) pi / 2 ~ 2.7
    assert mse < bound
    # Lloyd-Max is optimal: any perturbed codebook (with its own midpoints) is worse
    rng = np.random.default_rng(0)
    for _ in range(20):
        c2 = np.sort(c + 1e-3 * rng.standard_normal(8))
        assert O.lloyd_max_mse(c2, 0.5 * (c2[:-1] + c2[1:])) > mse


# ----------------------------------------------------------- value codec ---
def test_v_quantize_is_bruteforce_nearest_centroid():
    c, _ = O.codebook()
    rng = np.random.default_rng(3)
    x = rng.standard_normal(20000) * 1.5
    want = np.argmin(np.abs(x[:, None] - c[None, :]), axis=1)
    np.testing.assert_array_equal(O.v_quantize(x), want)
    # tie exactly on a threshold goes to the lower index (first minimum)
    assert O.v_quantize(np.array([0.0]))[0] == 3
    assert O.v_quantize(np.array([1e-12]))[0] == 4
    assert O.v_quantize(np.array([-10.0, 10.0])).tolist() == [0, 7]


def test_v_codec_statistics_on_gaussian_input():
    c, t = O.codebook()
    rng = np.random.default_rng(11)
    d = 128
    V = rng.standard_normal((8192, d)).astype(np.float16)
    idx, v_rot = O.v_encode(V)
    V64 = V.astype(np.float64)
    # rotation is orthonormal: rotated coordinates are again N(0,1)
    assert abs(np.mean(v_rot ** 2) / np.mean(V64 ** 2) - 1) < 1e-12
    # per-coordinate MSE in the rotated domain = the Lloyd-Max MSE, and it carries over unchanged
    # to the original domain through the inverse rotation (Parseval)
    mse_rot = np.mean((c[idx] - v_rot) ** 2)
    mse_orig = np.mean((O.v_decode(idx) - V64) ** 2)
    expect = O.lloyd_max_mse(c, t)
    assert abs(mse_rot / expect - 1) < 0.01
    assert abs(mse_orig / mse_rot - 1) < 1e-9
    assert mse_orig < O.turboquant_mse_bound(3)
    # code histogram = cell probabilities of N(0,1)
    edges = np.array([-np.inf, *t, np.inf])
    probs = np.diff(scipy.stats.norm.cdf(edges))
    hist = np.bincount(idx.ravel(), minlength=8) / idx.size
    np.testing.assert_allclose(hist, probs, atol=2e-3)


def test_v_decode_inverts_rotation_exactly_when_no_quantization_error():
    # a vector whose rotated coordinates ARE centroids must come back exactly:
    # pins the 1/sqrt(d) (not 1/d) inverse scaling and the transform direction.
    c, _ = O.codebook()
    rng = np.random.default_rng(5)
    for d in (64, 128):
        idx = rng.integers(0, 8, size=(6, d)).astype(np.uint8)
        v = scipy.linalg.hadamard(d) @ c[idx].T / math.sqrt(d)     # dense inverse, library matrix
        np.testing.assert_allclose(O.v_decode(idx), v.T, atol=1e-12)
        np.testing.assert_allclose(O.v_rotate(v.T), c[idx], atol=1e-12)
        np.testing.assert_array_equal(O.v_quantize(O.v_rotate(v.T)), idx)


def test_v_encode_single_spike_and_constant_vectors():
    # closed forms: e_j -> row j of H / sqrt(d) (all +-1/sqrt(d)); constant a -> a*sqrt(d) e_0
    d = 64
    v = np.zeros((1, d), dtype=np.float16); v[0, 5] = 8.0
    idx, v_rot = O.v_encode(v)
    signs = np.array([(-1) ** bin(i & 5).count("1") for i in range(d)])
    np.testing.assert_allclose(v_rot[0], signs * 1.0)              # 8/sqrt(64) = 1
    assert set(idx[0].tolist()) == {2, 5}                          # +-1.0 -> centroids +-0.756
    v = np.full((1, d), 0.25, dtype=np.float16)
    idx, v_rot = O.v_encode(v)
    assert v_rot[0, 0] == 2.0 and np.all(v_rot[0, 1:] == 0.0)
    assert idx[0, 0] == 7 and np.all(idx[0, 1:] == 3)              # 2.0 > 1.748 ; exact 0 -> lower


# --------------------------------------------------------------- packing ---
def test_pack_layout_hand_computed():
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 0]], dtype=np.uint8)
    c = codes[0].tolist()
    b0 = (c[0] | c[1] << 3 | (c[2] & 3) << 6) & 0xFF
    b1 = (c[2] >> 2 | c[3] << 1 | c[4] << 4 | (c[5] & 1) << 7) & 0xFF
    b2 = (c[5] >> 1 | c[6] << 2 | c[7] << 5) & 0xFF
    assert O.v_pack(codes).tolist() == [[b0, b1, b2]]
    assert O.v_pack(np.zeros((2, 64), np.uint8)).shape == (2, 24)
    assert O.v_pack(np.zeros((2, 128), np.uint8)).shape == (2, 48)


def test_pack_unpack_exhaustive_one_group():
    # all 8^8 code patterns of one 3-byte group, in chunks
    base = np.array(list(itertools.product(range(8), repeat=4)), dtype=np.uint8)   # 4096 x 4
    seen = set()
    for hi in range(0, 4096, 512):
        a = np.repeat(base[hi:hi + 512], 4096, axis=0)
        b = np.tile(base, (512, 1))
        codes = np.concatenate([a, b], axis=1)
        packed = O.v_pack(codes)
        assert packed.shape == (codes.shape[0], 3)
        np.testing.assert_array_equal(O.v_unpack(packed, 8), codes)
        word = packed[:, 0].astype(np.uint32) | packed[:, 1].astype(np.uint32) << 8 \
            | packed[:, 2].astype(np.uint32) << 16
        seen.add(int(word.min())); seen.add(int(word.max()))
        assert np.unique(word).size == codes.shape[0]             # injective
    assert 0 in seen and (1 << 24) - 1 in seen


# ------------------------------------------------------------------ q8_0 ---
def _rand_k(rng, shape):
    k = rng.standard_normal(shape) * np.exp(0.7 * rng.standard_normal(shape[:-1] + (1,)))
    return k.astype(np.float16)


def test_q8_error_bound_and_extremes():
    rng = np.random.default_rng(21)
    K = _rand_k(rng, (3, 50, 128))
    q, s, _ = O.k_encode(K)
    assert q.dtype == np.int8 and s.dtype == np.float16 and s.shape == (3, 50, 4)
    kh = O.k_decode(q, s)
    sb = np.repeat(s.astype(np.float64), 32, axis=-1)
    err = np.abs(kh - K.astype(np.float64))
    assert np.all(err <= sb / 2 * (1 + 1e-6))                      # half a step
    # the block maximum maps to +-127 and nothing clips at -128
    kb = np.abs(K.astype(np.float64)).reshape(3, 50, 4, 32)
    qb = np.abs(q.astype(np.int32)).reshape(3, 50, 4, 32)
    assert np.all(qb.max(-1) == 127)
    assert np.all(np.take_along_axis(qb, kb.argmax(-1)[..., None], -1) == 127)
    assert q.min() >= -127
    # stored scale is amax/127 to fp16 accuracy
    np.testing.assert_allclose(s.astype(np.float64) * 127, kb.max(-1), rtol=2.0 ** -11)


def test_q8_codes_are_bruteforce_nearest_multiples_of_stored_scale():
    rng = np.random.default_rng(22)
    K = _rand_k(rng, (40, 64))
    q, s, pre = O.k_encode(K)
    sb = np.repeat(s.astype(np.float64), 32, axis=-1)
    cand = np.arange(-128, 128, dtype=np.float64)
    dist = np.abs(K.astype(np.float64)[..., None] - cand * sb[..., None])
    best = dist.min(-1)
    got = np.abs(K.astype(np.float64) - q * sb)
    # the chosen code is a nearest one, except where fp32 rounding of k/s sits on a .5 tie
    near_tie = np.abs(np.abs(pre - np.floor(pre)) - 0.5) < 1e-4
    assert np.all((got <= best * (1 + 1e-9) + 1e-12) | near_tie)
    assert near_tie.mean() < 0.01


def test_q8_special_blocks_and_scale_invariance():
    z = np.zeros((2, 64), dtype=np.float16)
    q, s, _ = O.k_encode(z)
    assert not q.any() and not s.any()
    assert not O.k_decode(q, s).any()
    const = np.full((1, 32), -0.375, dtype=np.float16)
    q, s, _ = O.k_encode(const)
    assert np.all(q == -127)
    one = np.zeros((1, 32), dtype=np.float16); one[0, 9] = 3.0
    q, s, _ = O.k_encode(one)
    assert q[0, 9] == 127 and np.count_nonzero(q) == 1
    rng = np.random.default_rng(23)
    K = rng.standard_normal((16, 128)).astype(np.float16)
    q1, s1, _ = O.k_encode(K)
    q2, s2, _ = O.k_encode((K.astype(np.float32) * 4).astype(np.float16))   # exact power-of-two scaling
    np.testing.assert_array_equal(q1, q2)
    np.testing.assert_array_equal(s1.astype(np.float32) * 4, s2.astype(np.float32))
    # ties round to even: with s = 1 (amax = 127) the values 0.5, 1.5, 2.5 are exact ties
    blk = np.zeros((1, 32), dtype=np.float16)
    blk[0, :5] = [127.0, 0.5, 1.5, 2.5, -0.5]
    q, s, _ = O.k_encode(blk)
    assert float(s[0, 0]) == 1.0 and q[0, :5].tolist() == [127, 0, 2, 2, 0]


def test_q8_per_tensor_form_of_the_papers_formula():
    rng = np.random.default_rng(24)
    K = rng.standard_normal((2, 3, 10, 64)).astype(np.float16)
    q, s, _ = O.k_encode(K, block=None)
    assert s.shape == ()
    amax = np.abs(K.astype(np.float64)).max()
    assert abs(float(s) * 127 / amax - 1) < 2.0 ** -11
    kh = O.k_decode(q, s, block=None)
    assert np.abs(kh - K.astype(np.float64)).max() <= float(s) / 2 * (1 + 1e-6)
    assert np.abs(q.astype(np.int32)).max() == 127
    # one block of 32 is the same thing as the per-tensor form on that block
    blk = K[0, 0, 0, :32]
    qa, sa, _ = O.k_encode(blk[None, :])
    qb, sb_, _ = O.k_encode(blk, block=None)
    np.testing.assert_array_equal(qa[0], qb)
    assert sa[0, 0] == sb_


# ------------------------------------------------------------ byte counts ---
def test_compression_accounting_matches_paper():
    consts = {r[0]: float(r[1]) for r in read_golden_rows("paper_constants.txt")}
    b = O.stored_bytes(32, 8, 7194, 128)
    assert round(b["ratio_payload"], 2) == consts["compression_ratio"]
    assert b["dense16"] == 32 * 8 * 7194 * 128 * 2 * 2
    assert b["packed"] == 32 * 8 * 7194 * 184                      # 128 + 8 + 48 bytes per token-head
    assert abs(b["ratio_stored"] - 64 / 23) < 1e-12
    # payload-only bytes give exactly 16/5.5
    assert abs(b["dense16"] / (b["k_codes"] + b["v_codes"]) - 16 / 5.5) < 1e-12
    b64 = O.stored_bytes(1, 4, 600, 64)
    assert b64["packed"] == 4 * 600 * 92 and b64["dense16"] == 614400
    # the paper's memory table: N dense caches / one pool = N * (its measured ratio ~ 2.91)
    for agents, _tok, without, with_ in read_golden_rows("paper_memory_table.txt"):
        ratio = float(without) / int(agents) / float(with_)
        assert abs(ratio - consts["compression_ratio"]) < 0.01


# -------------------------------------------------------------- attention ---
def _naive_attention(q, Ks, Vs, scale):
    T, d = len(Ks), len(q)
    s = [scale * sum(q[j] * Ks[t][j] for j in range(d)) for t in range(T)]
    m = max(s)
    w = [math.exp(x - m) for x in s]
    z = sum(w)
    return [sum(w[t] * Vs[t][j] for t in range(T)) / z for j in range(d)]


def test_attend_matches_pure_python_bruteforce_with_gqa_and_tails():
    rng = np.random.default_rng(31)
    L, H, T, d, A, nq, qh = 2, 2, 9, 8, 3, 2, 4
    Kh = rng.standard_normal((L, H, T, d))
    Vh = rng.standard_normal((L, H, T, d))
    Q = rng.standard_normal((L, A, nq, qh, d))
    tails = [None,
             (rng.standard_normal((L, H, 3, d)).astype(np.float16),
              rng.standard_normal((L, H, 3, d)).astype(np.float16)),
             (np.zeros((L, H, 0, d), np.float16), np.zeros((L, H, 0, d), np.float16))]
    out = O.pool_attend(Kh, Vh, Q, tails=tails)
    assert out.shape == Q.shape
    for l in range(L):
        for a in range(A):
            for i in range(nq):
                for h in range(qh):
                    kv = h // 2
                    Ks = Kh[l, kv].tolist(); Vs = Vh[l, kv].tolist()
                    if a == 1:
                        Ks += tails[1][0][l, kv].astype(np.float64).tolist()
                        Vs += tails[1][1][l, kv].astype(np.float64).tolist()
                    want = _naive_attention(Q[l, a, i, h].tolist(), Ks, Vs, 1 / math.sqrt(d))
                    np.testing.assert_allclose(out[l, a, i, h], want, rtol=1e-12, atol=1e-13)


def test_attend_special_cases_and_agent_count_invariance():
    rng = np.random.default_rng(32)
    L, H, T, d = 1, 2, 40, 16
    Vh = rng.standard_normal((L, H, T, d))
    Q = rng.standard_normal((L, 4, 1, 2, d))
    # zero keys -> uniform weights -> mean of the values
    out = O.pool_attend(np.zeros((L, H, T, d)), Vh, Q)
    np.testing.assert_allclose(out[0, 2, 0, 1], Vh[0, 1].mean(0), atol=1e-13)
    # one dominant key -> its value
    Kh = np.zeros((L, H, T, d)); Kh[0, 0, 17] = 200.0 * Q[0, 0, 0, 0]
    out = O.pool_attend(Kh, Vh, Q)
    np.testing.assert_allclose(out[0, 0, 0, 0], Vh[0, 0, 17], atol=1e-9)
    # an agent's result does not depend on which other agents are batched with it
    Kh = rng.standard_normal((L, H, T, d))
    full = O.pool_attend(Kh, Vh, Q)
    alone = O.pool_attend(Kh, Vh, Q[:, 2:3])
    np.testing.assert_array_equal(full[:, 2:3], alone)
    # explicit scale argument
    np.testing.assert_allclose(O.pool_attend(Kh, Vh, Q, scale=0.25), O.pool_attend(Kh, Vh, Q))


def test_end_to_end_pool_roundtrip_and_linearity_of_rotation():
    rng = np.random.default_rng(33)
    L, H, T, d = 1, 2, 33, 64
    K = rng.standard_normal((L, H, T, d)).astype(np.float16)
    V = rng.standard_normal((L, H, T, d)).astype(np.float16)
    pool = O.pool_encode(K, V)
    assert pool["v_packed"].shape == (L, H, T, 24) and pool["k_scales"].shape == (L, H, T, 2)
    Kh, Vh = O.pool_decode(pool)
    assert np.abs(Kh - K.astype(np.float64)).max() < 0.03
    assert np.mean((Vh - V.astype(np.float64)) ** 2) < O.turboquant_mse_bound(3)
    # weighting centroids first and rotating once equals rotating every token then weighting
    c, _ = O.codebook()
    p = rng.random(T); p /= p.sum()
    once = O.fwht(p @ c[pool["v_idx"][0, 1]]) / math.sqrt(d)
    np.testing.assert_allclose(once, p @ Vh[0, 1], atol=1e-13)


def test_causal_tail_attention_equals_dense_masked_attention():
    """Multi-token decode step: query i of an agent sees the pool and the tail up to its own position.
    Checked against a dense masked softmax written independently (one score matrix, one mask)."""
    rng = np.random.default_rng(11)
    L, H, T, d, A, nq, G = 1, 2, 9, 16, 2, 3, 2
    Kp = rng.standard_normal((L, H, T, d))
    Vp = rng.standard_normal((L, H, T, d))
    Q = rng.standard_normal((L, A, nq, H * G, d))
    lens = [5, 1]                     # agent 1: shorter than nq - 1, so its first query sees no tail token
    tails = [(rng.standard_normal((L, H, n, d)), rng.standard_normal((L, H, n, d))) for n in lens]
    out = O.pool_attend(Kp, Vp, Q, tails=tails, tail_causal=True)
    for a in range(A):
        t_a = lens[a]
        for h in range(H * G):
            kv = h // G
            Kall = np.concatenate([Kp[0, kv], tails[a][0][0, kv]], axis=0)
            Vall = np.concatenate([Vp[0, kv], tails[a][1][0, kv]], axis=0)
            S = Q[0, a, :, h] @ Kall.T / np.sqrt(d)                           # [nq, T + t_a]
            pos = np.arange(T + t_a)[None, :]
            allowed = pos < (T + t_a - (nq - 1 - np.arange(nq)))[:, None]     # query i: all but the last nq-1-i
            allowed |= pos < T                                                # the pool is always visible
            S = np.where(allowed, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            np.testing.assert_allclose(out[0, a, :, h], P @ Vall, rtol=1e-12, atol=1e-12)
    # the last query sees everything; with one query per agent the flag changes nothing
    full = O.pool_attend(Kp, Vp, Q, tails=tails)
    np.testing.assert_array_equal(out[:, :, -1], full[:, :, -1])
    np.testing.assert_array_equal(O.pool_attend(Kp, Vp, Q[:, :, :1], tails=tails, tail_causal=True),
                                  O.pool_attend(Kp, Vp, Q[:, :, :1], tails=tails))


# ------------------------------------------------ value codec, scaled variant ---
def test_scaled_values_closed_forms():
    c, _ = O.codebook()
    d = 64
    # constant vector a: rms = a, rotated = a*sqrt(d) e_0 -> code 7 at coordinate 0, exact zeros elsewhere
    v = np.full((1, d), 0.75, dtype=np.float16)
    idx, g16, v_rot, rms = O.v_encode_scaled(v)
    assert rms[0] == 0.75 and g16[0] == np.float16(0.75)
    assert idx[0, 0] == 7 and np.all(idx[0, 1:] == 3)
    # decode, by a dense library matrix: g * H c[idx] / sqrt(d)
    want = 0.75 * (scipy.linalg.hadamard(d) @ c[idx[0]]) / math.sqrt(d)
    np.testing.assert_allclose(O.v_decode_scaled(idx, g16)[0], want, atol=1e-12)
    # one spike a e_j: rms = a/sqrt(d); rotated coordinates +-a/sqrt(d) = +-1 in units of the scale
    v = np.zeros((1, d), dtype=np.float16); v[0, 9] = 4.0
    idx, g16, v_rot, rms = O.v_encode_scaled(v)
    assert rms[0] == 0.5 and g16[0] == np.float16(0.5)
    signs = np.array([(-1) ** bin(i & 9).count("1") for i in range(d)])
    np.testing.assert_array_equal(idx[0], np.where(signs > 0, 5, 2))   # +-1.0 -> centroids +-0.756
    # zero scale (the zero vector, or one too short for fp16): the codes of the zero vector, decodes to zero
    tiny = np.zeros((2, d), dtype=np.float16); tiny[1, 3] = 6e-8
    idx, g16, _, rms = O.v_encode_scaled(tiny)
    assert rms[1] > 0 and np.all(g16 == 0) and np.all(idx == 3) and np.all(O.v_decode_scaled(idx, g16) == 0)
    assert np.array_equal(idx[0], O.v_encode(tiny[:1])[0][0])
    # the format limit: scales above 128 are stored as 128
    v = np.full((1, d), 300.0, dtype=np.float16)
    idx, g16, _, rms = O.v_encode_scaled(v)
    assert rms[0] == 300.0 and g16[0] == np.float16(128.0)


def test_scaled_values_are_the_unscaled_codec_on_the_normalized_vector():
    # dividing by the stored scale and running the paper's own value quantizer gives the same codes
    # (wherever the division does not land within rounding of a threshold)
    rng = np.random.default_rng(21)
    d = 128
    sigma = np.exp(rng.normal(0.0, 1.5, size=(512, 1)))
    V = (rng.standard_normal((512, d)) * sigma).astype(np.float16)
    idx, g16, v_rot, rms = O.v_encode_scaled(V)
    g = g16.astype(np.float64)[:, None]
    u = v_rot / g
    _, t = O.codebook()
    near = np.min(np.abs(u[..., None] - t), axis=-1) < 1e-9
    assert np.array_equal(O.v_quantize(u)[~near], idx[~near])
    # rms is ||v|| / sqrt(d), by the library norm, and the stored scale is its fp16 rounding
    np.testing.assert_allclose(rms, np.linalg.norm(V.astype(np.float64), axis=-1) / math.sqrt(d), rtol=1e-14)
    np.testing.assert_array_equal(g16, rms.astype(np.float16))
    assert abs(np.mean(u ** 2) - 1) < 1e-3                          # unit-variance coordinates


def test_scaled_values_scale_invariance_and_distortion():
    c, t = O.codebook()
    rng = np.random.default_rng(22)
    d = 128
    base = rng.standard_normal((4096, d)).astype(np.float16)
    idx1, g1, _, _ = O.v_encode_scaled(base)
    for k in (-6, 3, 5):                                            # powers of two: exact in fp16
        Vk = (base.astype(np.float32) * 2.0 ** k).astype(np.float16)
        idxk, gk, _, _ = O.v_encode_scaled(Vk)
        np.testing.assert_array_equal(idxk, idx1)
        np.testing.assert_array_equal(gk.astype(np.float64), g1.astype(np.float64) * 2.0 ** k)
    # relative distortion = the Lloyd-Max MSE of N(0,1), whatever the vectors' lengths; it meets the
    # bound of section "TurboQuant".  The unscaled codec on the same data does not.
    sigma = np.exp(rng.normal(0.0, 1.0, size=(4096, 1)))
    V = (base.astype(np.float64) * sigma).astype(np.float16)
    V64 = V.astype(np.float64)
    idx, g16, _, _ = O.v_encode_scaled(V)
    rel = np.sum((O.v_decode_scaled(idx, g16) - V64) ** 2, axis=-1) / np.sum(V64 ** 2, axis=-1)
    assert abs(np.mean(rel) / O.lloyd_max_mse(c, t) - 1) < 0.02
    assert np.mean(rel) < O.turboquant_mse_bound(3)
    idx0, _ = O.v_encode(V)
    rel0 = np.sum((O.v_decode(idx0) - V64) ** 2, axis=-1) / np.sum(V64 ** 2, axis=-1)
    assert np.mean(rel0) > 2 * np.mean(rel)


def test_scaled_values_match_turboquant_on_unit_vectors():
    # TurboQuant's statement (section "TurboQuant"): a unit vector's rotated coordinates are ~N(0, 1/d)
    # and are quantized with the N(0,1) codebook scaled by 1/sqrt(d).  Brute-force nearest centroid.
    c, t = O.codebook()
    rng = np.random.default_rng(23)
    d = 128
    x = rng.standard_normal((256, d))
    x /= np.linalg.norm(x, axis=-1, keepdims=True)
    V = (x * 64.0).astype(np.float16)                               # any length: only the direction matters
    idx, g16, v_rot, rms = O.v_encode_scaled(V)
    unit_rot = v_rot / (rms[:, None] * math.sqrt(d))                # rotation of v/||v||
    want = np.argmin(np.abs(unit_rot[..., None] - c / math.sqrt(d)), axis=-1)
    # the stored scale is rms rounded to fp16 (relative 2^-11): codes may differ only that close to a threshold
    near = np.min(np.abs(unit_rot[..., None] * math.sqrt(d) - t), axis=-1) < 2.2 * 2.0 ** -11
    assert np.array_equal(want[~near], idx[~near])
    assert near.mean() < 0.01


def test_scaled_values_pool_roundtrip_and_bytes():
    rng = np.random.default_rng(24)
    K = rng.standard_normal((1, 2, 40, 64)).astype(np.float16)
    V = (rng.standard_normal((1, 2, 40, 64)) * 3.0).astype(np.float16)
    ref = O.pool_encode(K, V, scaled_values=True)
    assert ref["v_scales"].shape == (1, 2, 40) and ref["v_scales"].dtype == np.float16
    Kh, Vh = O.pool_decode(ref)
    np.testing.assert_array_equal(Vh, O.v_decode_scaled(ref["v_idx"], ref["v_scales"]))
    assert np.mean((Vh - V.astype(np.float64)) ** 2) / np.mean(V.astype(np.float64) ** 2) < 0.05
    b = O.stored_bytes(32, 8, 4096, 128, scaled_values=True)
    assert b["packed"] == 32 * 8 * 4096 * 186 and abs(b["ratio_stored"] - 512 / 186) < 1e-12


# ------------------------------------------------ value codec, int8 variant ---
def test_int8_values_error_bound_extremes_and_bruteforce():
    rng = np.random.default_rng(31)
    d = 128
    V = (rng.standard_normal((300, d)) * np.exp(rng.standard_normal((300, 1)))).astype(np.float16)
    q, s, pre = O.v_encode_int8(V)
    assert q.dtype == np.int8 and s.dtype == np.float16 and s.shape == (300,)
    V64, s64 = V.astype(np.float64), s.astype(np.float64)
    # one scale per vector = max|v|/127 to fp16 accuracy; the maximum maps to +-127; half-step error
    np.testing.assert_allclose(s64 * 127, np.abs(V64).max(-1), rtol=2.0 ** -11)
    assert np.all(np.abs(q.astype(np.int32)).max(-1) == 127) and q.min() >= -127
    assert np.all(np.abs(O.v_decode_int8(q, s) - V64) <= s64[:, None] / 2 * (1 + 1e-6))
    # brute force: the code is a nearest multiple of the stored scale (fp32 ties aside)
    cand = np.arange(-128, 128, dtype=np.float64)
    best = np.abs(V64[:40, :, None] - cand * s64[:40, None, None]).min(-1)
    got = np.abs(V64[:40] - q[:40] * s64[:40, None])
    near_tie = np.abs(np.abs(pre[:40] - np.floor(pre[:40])) - 0.5) < 1e-4
    assert np.all((got <= best * (1 + 1e-9) + 1e-12) | near_tie) and near_tie.mean() < 0.01
    # no rotation: a spike stays a spike, a constant stays a constant
    one = np.zeros((1, d), dtype=np.float16); one[0, 9] = -3.0
    q1, s1, _ = O.v_encode_int8(one)
    assert q1[0, 9] == -127 and np.count_nonzero(q1) == 1 and O.v_decode_int8(q1, s1)[0, 9] == -127 * float(s1[0])
    z, sz, _ = O.v_encode_int8(np.zeros((1, d), dtype=np.float16))
    assert not z.any() and sz[0] == 0 and not O.v_decode_int8(z, sz).any()
    # power-of-two scale invariance; ties to even with s = 1
    q2, s2, _ = O.v_encode_int8((V.astype(np.float32) * 8).astype(np.float16))
    np.testing.assert_array_equal(q2, q)
    np.testing.assert_array_equal(s2.astype(np.float32), s.astype(np.float32) * 8)
    blk = np.zeros((1, d), dtype=np.float16); blk[0, :5] = [127.0, 0.5, 1.5, 2.5, -0.5]
    qt, st, _ = O.v_encode_int8(blk)
    assert float(st[0]) == 1.0 and qt[0, :5].tolist() == [127, 0, 2, 2, 0]


def test_int8_values_scale_cap_and_pool_roundtrip():
    d = 64
    v = np.zeros((1, d), dtype=np.float16)
    v[0, :4] = [40000.0, -40000.0, 16256.0, 130.0]                  # 40000/127 > 128: the cap acts
    q, s, _ = O.v_encode_int8(v)
    assert float(s[0]) == 128.0 and q[0, :4].tolist() == [127, -128, 127, 1]
    v[0, :2] = [16256.0, -16256.0]                                  # exactly at the cap: 16256/127 = 128
    q, s, _ = O.v_encode_int8(v)
    assert float(s[0]) == 128.0 and q[0, :3].tolist() == [127, -127, 127]
    rng = np.random.default_rng(32)
    K = rng.standard_normal((1, 2, 40, d)).astype(np.float16)
    V = (rng.standard_normal((1, 2, 40, d)) * 3.0).astype(np.float16)
    ref = O.pool_encode(K, V, int8_values=True)
    assert ref["v_codes"].shape == V.shape and ref["v_scales"].shape == (1, 2, 40)
    Kh, Vh = O.pool_decode(ref)
    np.testing.assert_array_equal(Vh, ref["v_codes"].astype(np.float64) * ref["v_scales"].astype(np.float64)[..., None])
    assert np.abs(Vh - V.astype(np.float64)).max() <= float(ref["v_scales"].max()) / 2 * (1 + 1e-6)
    b = O.stored_bytes(32, 8, 4096, 128, int8_values=True)
    assert b["packed"] == 32 * 8 * 4096 * (136 + 130) and abs(b["ratio_stored"] - 512 / 266) < 1e-12
    # with head_dim 32 a vector is one q8_0 block: the key quantizer, re-called through its own entry point
    V32 = rng.standard_normal((50, 32)).astype(np.float16)
    qa, sa, _ = O.v_encode_int8(V32)
    qb, sb, _ = O.k_encode(V32)
    np.testing.assert_array_equal(qa, qb)
    np.testing.assert_array_equal(sa, sb[:, 0])


# ------------------------------------------------------------ bfloat16 inputs ---
def test_bfloat16_inputs_same_quantizers_wider_range():
    from paper_2604_24971_amd import workloads as W
    rng = np.random.default_rng(41)
    x = (rng.standard_normal((64, 128)) * np.exp(2.0 * rng.standard_normal((64, 1)))).astype(np.float32)
    xb = W.bf16_round(x)
    # the rounding helper: representable, within half a bfloat16 step, idempotent, ties to even
    assert not np.any(xb.view(np.uint32) & 0xFFFF)
    assert np.all(np.abs(xb - x) <= np.abs(x) * 2.0 ** -8)
    np.testing.assert_array_equal(W.bf16_round(xb), xb)
    tie = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)      # halfway between neighbours
    np.testing.assert_array_equal(W.bf16_round(tie), np.array([1.0, 1.0 + 2.0 ** -6], dtype=np.float32))
    with pytest.raises(TypeError):
        O.k_encode(x)                                               # float32 that is not bfloat16
    with pytest.raises(TypeError):
        O.v_encode(x.astype(np.float64))
    # values that float16 also holds exactly give the same result through either dtype
    small = W.bf16_round(rng.standard_normal((8, 128)).astype(np.float32))
    qa, sa, _ = O.k_encode(small)
    qb, sb, _ = O.k_encode(small.astype(np.float16))
    np.testing.assert_array_equal(qa, qb); np.testing.assert_array_equal(sa, sb)
    np.testing.assert_array_equal(O.v_encode(small)[0], O.v_encode(small.astype(np.float16))[0])
    # the q8_0 invariants hold on bfloat16 data
    q, s, _ = O.k_encode(xb)
    sb_ = np.repeat(s.astype(np.float64), 32, axis=-1)
    assert np.all(np.abs(O.k_decode(q, s) - xb.astype(np.float64)) <= sb_ / 2 * (1 + 1e-6))
    assert np.all(np.abs(q.astype(np.int32)).reshape(64, 4, 32).max(-1) == 127)
    # beyond float16's range: the scale saturates at 65504 and the codes clip
    big = np.zeros((1, 32), dtype=np.float32); big[0, :3] = [2.0 ** 30, -2.0 ** 30, 3 * 2.0 ** 16]
    q, s, _ = O.k_encode(big)
    assert float(s[0, 0]) == 65504.0 and q[0, :3].tolist() == [127, -128, 3]
    tiny = np.zeros((1, 32), dtype=np.float32); tiny[0, 0] = 2.0 ** -40     # below float16: scale 0, codes 0
    q, s, _ = O.k_encode(tiny)
    assert float(s[0, 0]) == 0.0 and not q.any()


# ------------------------------------------------------- rotation with a sign diagonal ---
def test_sign_diagonal_generator_matches_published_splitmix64_vectors():
    for row in read_golden_rows("splitmix64_vectors.txt"):
        seed, want = int(row[0]), [int(x) for x in row[1:]]
        assert O.splitmix64(seed, len(want)) == want
    s = O.rotation_signs(1234567, 128)
    assert s.shape == (128,) and set(s.tolist()) == {-1.0, 1.0}
    # the first published outputs are odd, odd, odd, odd, odd -> five negated coordinates
    assert s[:5].tolist() == [-1.0] * 5
    assert 40 < (s < 0).sum() < 88                                  # about half
    assert np.all(O.rotation_signs(0, 64) == 1.0)                   # seed 0: the plain transform
    assert not np.array_equal(O.rotation_signs(1, 128), O.rotation_signs(2, 128))


def test_sign_diagonal_rotation_is_orthonormal_and_equals_the_dense_matrix():
    rng = np.random.default_rng(51)
    c, _ = O.codebook()
    for d in (64, 128):
        s = O.rotation_signs(99, d)
        x = rng.standard_normal((5, d)).astype(np.float16)
        R = scipy.linalg.hadamard(d) @ np.diag(s) / math.sqrt(d)    # library matrix: H D / sqrt(d)
        np.testing.assert_allclose(O.v_rotate(x, s), x.astype(np.float64) @ R.T, atol=1e-12)
        np.testing.assert_allclose(R @ R.T, np.eye(d), atol=1e-12)
        # decoding applies the inverse (= transpose): codes whose centroids ARE the rotated vector come back
        idx = rng.integers(0, 8, size=(4, d)).astype(np.uint8)
        v = c[idx] @ R                                              # R^T c, row-wise
        np.testing.assert_allclose(O.v_decode(idx, s), v, atol=1e-12)
        np.testing.assert_allclose(O.v_rotate(v, s), c[idx], atol=1e-12)
        g = np.full(4, 0.5, dtype=np.float16)
        np.testing.assert_allclose(O.v_decode_scaled(idx, g, s), 0.5 * v, atol=1e-12)


def test_sign_diagonal_keeps_structured_vectors_from_saturating():
    # a constant vector: the bare transform piles it onto coordinate 0 (2.15 is the largest centroid),
    # the signed one spreads it like a random vector
    d = 128
    V = np.full((1, d), 1.0, dtype=np.float16)
    plain = O.v_decode(O.v_encode(V)[0])
    s = O.rotation_signs(7, d)
    signed = O.v_decode(O.v_encode(V, s)[0], s)
    err_plain = np.mean((plain - 1.0) ** 2)
    err_signed = np.mean((signed - 1.0) ** 2)
    assert err_plain > 0.5 and err_signed < 0.08
    # through the pool functions, both rotating codecs
    rng = np.random.default_rng(52)
    K = rng.standard_normal((1, 1, 40, 64)).astype(np.float16)
    Vp = (1.0 + 0.05 * rng.standard_normal((1, 1, 40, 64))).astype(np.float16)
    for scaled in (False, True):
        a = O.pool_decode(O.pool_encode(K, Vp, scaled_values=scaled))[1]
        b = O.pool_decode(O.pool_encode(K, Vp, scaled_values=scaled, sign_seed=7))[1]
        V64 = Vp.astype(np.float64)
        assert np.mean((b - V64) ** 2) < 0.2 * np.mean((a - V64) ** 2)
    with pytest.raises(ValueError):
        O.pool_encode(K, Vp, int8_values=True, sign_seed=7)


# ------------------------------------------------ keys with one scale per layer tensor ---
def test_per_tensor_key_scale_pool_form_and_the_papers_ratio():
    rng = np.random.default_rng(61)
    L, H, T, d = 3, 2, 50, 64
    K = (rng.standard_normal((L, H, T, d)) * np.array([0.5, 2.0, 7.0])[:, None, None, None]).astype(np.float16)
    V = rng.standard_normal((L, H, T, d)).astype(np.float16)
    ref = O.pool_encode(K, V, key_per_tensor=True)
    assert ref["k_scales"].shape == (L,) and ref["k_scales"].dtype == np.float16
    K64 = K.astype(np.float64)
    for l in range(L):
        amax = np.abs(K64[l]).max()
        s = float(ref["k_scales"][l])
        assert abs(s * 127 / amax - 1) < 2.0 ** -11                   # s = max|K| / 127 over the layer tensor
        assert np.abs(ref["k_codes"][l].astype(np.int32)).max() == 127
        # brute force: every code is a nearest multiple of that one scale
        cand = np.arange(-128, 128, dtype=np.float64) * s
        best = np.abs(K64[l][..., None] - cand).min(-1)
        got = np.abs(K64[l] - ref["k_codes"][l] * s)
        near_tie = np.abs(np.abs(ref["k_pre"][l] - np.floor(ref["k_pre"][l])) - 0.5) < 1e-4
        assert np.all((got <= best * (1 + 1e-9) + 1e-12) | near_tie)
    Kh, _ = O.pool_decode(ref)
    assert np.all(np.abs(Kh - K64) <= ref["k_scales"].astype(np.float64)[:, None, None, None] / 2 * (1 + 1e-6))
    # layers are independent tensors: encoding one layer alone gives the same codes
    one = O.pool_encode(K[1:2], V[1:2], key_per_tensor=True)
    np.testing.assert_array_equal(one["k_codes"][0], ref["k_codes"][1])
    # without per-block scales the stored bytes give exactly the ratio the paper states, 16 / 5.5
    consts = {r[0]: float(r[1]) for r in read_golden_rows("paper_constants.txt")}
    b = O.stored_bytes(32, 8, 7194, 128, key_per_tensor=True)
    assert b["packed"] == 32 * 8 * 7194 * 176 + 32 * 2
    assert round(b["ratio_stored"], 2) == consts["compression_ratio"]


# ------------------------------------------------------- other value bit widths ---
def test_codebooks_of_2_3_4_bits_match_the_published_table_and_the_bound():
    for row in read_golden_rows("max1960_table.txt"):
        levels, mse, want = int(row[0]), float(row[1]), np.array([float(x) for x in row[2:]])
        bits = levels.bit_length() - 1
        c, t = O.codebook(bits)
        assert c.shape == (levels,) and t.shape == (levels - 1,)
        np.testing.assert_allclose(c[levels // 2:], want, rtol=6e-4)      # four printed digits
        np.testing.assert_allclose(c, -c[::-1], atol=1e-15)
        assert abs(O.lloyd_max_mse(c, t) / mse - 1) < 1e-3
        assert O.lloyd_max_mse(c, t) < O.turboquant_mse_bound(bits)
        # fixed point, by numerical integration
        pdf = scipy.stats.norm.pdf
        edges = [-np.inf, *t, np.inf]
        for k in range(levels):
            mass = scipy.integrate.quad(pdf, edges[k], edges[k + 1])[0]
            mean = scipy.integrate.quad(lambda x: x * pdf(x), edges[k], edges[k + 1])[0] / mass
            assert abs(mean - c[k]) < 1e-8


@pytest.mark.parametrize("bits", [2, 4])
def test_value_codec_at_other_bit_widths(bits):
    c, t = O.codebook(bits)
    rng = np.random.default_rng(70 + bits)
    x = rng.standard_normal(20000) * 1.5
    np.testing.assert_array_equal(O.v_quantize(x, bits), np.argmin(np.abs(x[:, None] - c[None, :]), axis=1))
    assert O.v_quantize(np.array([0.0]), bits)[0] == (1 << bits) // 2 - 1    # a tie goes to the lower index
    # exhaustive pack / unpack of one byte-aligned group, and a hand-computed byte
    per = 8 // bits
    allc = np.array(list(itertools.product(range(1 << bits), repeat=per)), dtype=np.uint8)
    packed = O.v_pack(allc, bits)
    assert packed.shape == (allc.shape[0], 1)
    np.testing.assert_array_equal(O.v_unpack(packed, per, bits), allc)
    if bits == 4:
        assert O.v_pack(np.array([[0x3, 0xA]], dtype=np.uint8), 4)[0, 0] == 0xA3      # code 0 in the low nibble
    else:
        assert O.v_pack(np.array([[1, 2, 3, 0]], dtype=np.uint8), 2)[0, 0] == 0b00111001
    # statistics on Gaussian data: per-coordinate MSE = the codebook's, carried through the rotation
    d = 128
    V = rng.standard_normal((4096, d)).astype(np.float16)
    idx, v_rot = O.v_encode(V, bits=bits)
    assert idx.max() == (1 << bits) - 1
    mse = np.mean((O.v_decode(idx, bits=bits) - V.astype(np.float64)) ** 2)
    assert abs(mse / O.lloyd_max_mse(c, t) - 1) < 0.02
    # scaled variant and pool functions
    sig = np.exp(rng.standard_normal((4096, 1)))
    Vw = (V.astype(np.float64) * sig).astype(np.float16)
    idx, g16, _, _ = O.v_encode_scaled(Vw, bits=bits)
    rel = np.sum((O.v_decode_scaled(idx, g16, bits=bits) - Vw.astype(np.float64)) ** 2, -1) / np.sum(Vw.astype(np.float64) ** 2, -1)
    assert abs(rel.mean() / O.lloyd_max_mse(c, t) - 1) < 0.03
    assert np.all(O.v_encode_scaled(np.zeros((1, d), np.float16), bits=bits)[0] == (1 << bits) // 2 - 1)
    K = rng.standard_normal((1, 2, 40, 64)).astype(np.float16)
    Vp = rng.standard_normal((1, 2, 40, 64)).astype(np.float16)
    ref = O.pool_encode(K, Vp, value_bits=bits)
    assert ref["v_packed"].shape == (1, 2, 40, 64 * bits // 8) and ref["v_bits"] == bits
    _, Vh = O.pool_decode(ref)
    np.testing.assert_array_equal(Vh, O.v_decode(ref["v_idx"], bits=bits))
    assert O.stored_bytes(32, 8, 4096, 128, value_bits=bits)["packed"] == 32 * 8 * 4096 * (136 + 16 * bits)


def test_fp16_key_reading_rounds_once_to_nearest_even():
    """keys_as_fp16 (the cast of section "DynamicCache Injection", read as fp16): hand-computed roundings --
    fp16 has 11 significant bits, so 2049 is a tie (-> 2048, even), 2051 a tie (-> 2052), 2050 exact; values
    below 2^-24 / 2 vanish; the result of q8_0 dequantization code * s (up to 18 bits) loses at most half an ulp."""
    x = np.array([2049.0, 2050.0, 2051.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -0.1, 2.0 ** -26, 65504.0])
    want = np.array([2048.0, 2050.0, 2052.0, 1.0, 1.0 + 2.0 ** -9, -0.0999755859375, 0.0, 65504.0])
    np.testing.assert_array_equal(O.keys_as_fp16(x), want)
    rng = np.random.default_rng(5)
    K = (rng.standard_normal((1, 2, 50, 64)) * 6).astype(np.float16)
    ref = O.pool_encode(K, K)
    Kh, _ = O.pool_decode(ref)
    K16 = O.keys_as_fp16(Kh)
    assert np.all(np.abs(K16 - Kh) <= 2.0 ** -11 * np.abs(Kh) + 2.0 ** -25)
    assert np.any(K16 != Kh)                     # the products really have more than 11 bits
    # keys that fp16 holds exactly (scale a power of two: block maximum 127 * 2^k) pass unchanged
    K2 = np.zeros((1, 1, 4, 32), dtype=np.float16)
    K2[..., 0] = 127 * 0.25
    K2[..., 1:] = rng.integers(-127, 128, size=(1, 1, 4, 31)) * 0.25
    Kh2, _ = O.pool_decode(O.pool_encode(K2, K2))
    np.testing.assert_array_equal(O.keys_as_fp16(Kh2), Kh2)
