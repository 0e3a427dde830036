"""CPU oracle for the PolyKV shared-pool hot path.  TEST INFRASTRUCTURE ONLY.

This module is the plain, slow, obviously-correct statement of what the GPU
library computes.  It is imported only by tests, by the smoke check and by the
benchmark's CPU-baseline leg; the product path never touches it, and it shares
no code, tables or constants with the HIP sources (it derives its own codebook).

What it follows (PolyKV paper, section "Compression Scheme" unless noted):
  * Key quantization "q8_0":  s = max|K|/127,  Kq = clip(round(K/s), -128, 127),
    K_dequant = Kq * s.  The scale is taken per block of 32 consecutive head_dim
    elements (the block-32 reading of the q8_0 name); ``block=None`` gives the
    per-tensor form the paper's formula literally states.
  * Value quantization "TurboQuant MSE, 3-bit": V_rot = FWHT(V)/sqrt(d), then the
    nearest of the 8 Lloyd-Max centroids of N(0,1) (section "TurboQuant",
    paragraph "Lloyd-Max quantization"), indices bit-packed at 3 bits.
  * Dequantization (section "TurboQuant", paragraph "Dequantization"): look the
    centroids up and undo the rotation using H.H = d.I.  The forward transform is
    the normalized one, so the true inverse is H.c/sqrt(d); the paper's "divide by
    d" would return V/sqrt(d) and is read as the un-normalized-forward convention.
  * Read path: every agent's decode queries attend over the decoded pool (plus the
    agent's own full-precision continuation), standard scaled-dot-product softmax
    attention, grouped-query head mapping (section "Experimental Setup": Llama-3-8B
    uses GQA with 8 KV heads).

  * Variant "scaled values" (not in the PolyKV paper's steps; the TurboQuant analysis it cites in
    section "TurboQuant" assumes rotated coordinates of unit variance, which a raw cache does not
    have): a per-vector scale g = fp16(min(rms(v), 128)) is stored next to the codes, the thresholds
    and centroids are multiplied by g.  See v_encode_scaled.
  * Variant "int8 values": the uniform int8 value quantizer without rotation that the paper proposes
    as an ablation (sections "Discussion" hypothesis and "Future Work"): the key formula applied to
    each value vector with one scale per vector.  See v_encode_int8.
  * Variant "sign diagonal": the rotation is H.D instead of H, D a fixed diagonal of pseudorandom signs
    (the randomized-Hadamard construction of the rotation-based quantizers the paper discusses in
    section "Related Work"); it keeps structured vectors, which the bare transform maps to a few large
    coordinates, from saturating the codebook.  See rotation_signs.

Inputs: float16 arrays, or float32 arrays that stand for bfloat16 tensors (the paper's Llama-3-8B cache
is bfloat16, section "Experimental Setup") and must hold bfloat16-representable values.

Precision: float64 everywhere, except the steps whose float32/float16 rounding is
part of the stored format (the fp16 block scale and the code decision of q8_0).

Pins (tests/test_oracle_pins.py): H.H = d.I, Parseval and the dense Sylvester
matrix for the transform; the Lloyd-Max fixed-point conditions by numerical
integration and the centroid values the paper prints; the distortion bound; the
q8_0 half-step error bound; exhaustive pack/unpack; brute-force attention; byte
accounting for the 2.91x ratio.  Quality numbers of the paper (perplexity,
BERTScore) need model weights and texts and are: parity unpinned.
"""
from __future__ import annotations

import math

import numpy as np

Q8_BLOCK = 32          # elements per q8_0 block
V_BITS = 3             # bits per value code: the paper's choice; 2 and 4 are variants
V_LEVELS = 1 << V_BITS


# --------------------------------------------------------------------------- #
# Codebook: 8-level Lloyd-Max quantizer of the standard normal
# --------------------------------------------------------------------------- #
def _phi(x: float) -> float:
    return math.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi) if math.isfinite(x) else 0.0


def _Phi(x: float) -> float:
    if x == math.inf:
        return 1.0
    if x == -math.inf:
        return 0.0
    return 0.5 * (1.0 + math.erf(x / math.sqrt(2.0)))


def lloyd_max_gaussian(levels: int = V_LEVELS, tol: float = 1e-15, max_iter: int = 100000):
    """Centroids c[0..levels-1] (ascending) and thresholds t[0..levels-2] of the MSE-optimal
    scalar quantizer of N(0,1), by Lloyd's iteration: thresholds are midpoints of adjacent
    centroids, centroids are conditional means of their cells.
    (Section "TurboQuant", paragraph "Lloyd-Max quantization".)"""
    c = np.linspace(-2.0, 2.0, levels)
    for _ in range(max_iter):
        t = 0.5 * (c[:-1] + c[1:])
        edges = [-math.inf, *t.tolist(), math.inf]
        new = np.empty(levels)
        for k in range(levels):
            a, b = edges[k], edges[k + 1]
            new[k] = (_phi(a) - _phi(b)) / (_Phi(b) - _Phi(a))
        done = np.max(np.abs(new - c)) < tol
        c = new
        if done:
            break
    # enforce the exact odd symmetry the fixed point has
    c = 0.5 * (c - c[::-1])
    t = 0.5 * (c[:-1] + c[1:])
    return c, t


_CODEBOOKS = {}


def codebook(bits: int = V_BITS):
    """(centroids, thresholds) of the 2^bits-level quantizer (section "TurboQuant": b bits per coordinate;
    the paper uses b = 3)."""
    if bits not in _CODEBOOKS:
        _CODEBOOKS[bits] = lloyd_max_gaussian(1 << bits)
    return _CODEBOOKS[bits]


def lloyd_max_mse(c, t) -> float:
    """Per-coordinate MSE of the quantizer (c, t) on N(0,1):  sum_k  int_cell (x-c_k)^2 phi(x) dx,
    in closed form (second moment, first moment, mass of every cell)."""
    edges = [-math.inf, *np.asarray(t).tolist(), math.inf]
    total = 0.0
    for k, ck in enumerate(c):
        a, b = edges[k], edges[k + 1]
        mass = _Phi(b) - _Phi(a)
        m1 = _phi(a) - _phi(b)
        ax = a * _phi(a) if math.isfinite(a) else 0.0
        bx = b * _phi(b) if math.isfinite(b) else 0.0
        m2 = mass + ax - bx
        total += m2 - 2.0 * ck * m1 + ck * ck * mass
    return total


def turboquant_mse_bound(bits: int) -> float:
    """Distortion bound of section "TurboQuant", paragraph "Distortion bound"."""
    return math.sqrt(3.0) * math.pi / 2.0 / 4.0 ** bits


# --------------------------------------------------------------------------- #
# Walsh-Hadamard transform, natural (Sylvester) order, un-normalized
# --------------------------------------------------------------------------- #
def fwht(x):
    """y = H_d x along the last axis, H[i][j] = (-1)^popcount(i & j), float64 butterflies."""
    y = np.array(x, dtype=np.float64, copy=True)
    d = y.shape[-1]
    if d & (d - 1):
        raise ValueError("length must be a power of two")
    h = 1
    while h < d:
        z = y.reshape(y.shape[:-1] + (d // (2 * h), 2, h))
        a = z[..., 0, :].copy()
        b = z[..., 1, :].copy()
        z[..., 0, :] = a + b
        z[..., 1, :] = a - b
        h *= 2
    return y


# --------------------------------------------------------------------------- #
# Input tensors
# --------------------------------------------------------------------------- #
def _as_f32_input(X, name: str):
    """float16 -> float32 (exact); a float32 array is taken as a bfloat16 tensor and checked for it."""
    X = np.asarray(X)
    if X.dtype == np.float16:
        return X.astype(np.float32)
    if X.dtype == np.float32:
        if np.any(np.ascontiguousarray(X).view(np.uint32) & np.uint32(0xFFFF)):
            raise TypeError("%s: float32 input must hold bfloat16-representable values" % name)
        return X
    raise TypeError("%s must be float16, or float32 holding bfloat16 values" % name)


FP16_MAX = 65504.0


# --------------------------------------------------------------------------- #
# Sign diagonal of the rotation variant
# --------------------------------------------------------------------------- #
def splitmix64(seed: int, n: int):
    """The first n outputs of the SplitMix64 generator started at `seed` (Steele, Lea, Flood 2014): output
    i is the finalizer of seed + (i+1)*0x9E3779B97F4A7C15, so it can be computed per index."""
    mask = (1 << 64) - 1
    out = []
    for i in range(n):
        z = (seed + (i + 1) * 0x9E3779B97F4A7C15) & mask
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        out.append(z ^ (z >> 31))
    return out


def rotation_signs(seed: int, d: int):
    """Diagonal of D, float64 [d] of +-1: coordinate i is negated iff output i of splitmix64(seed) is odd.
    seed = 0 means no diagonal (the paper's plain transform)."""
    if seed == 0:
        return np.ones(d)
    return np.array([-1.0 if z & 1 else 1.0 for z in splitmix64(seed, d)])


# --------------------------------------------------------------------------- #
# Keys: q8_0
# --------------------------------------------------------------------------- #
def k_encode(K, block: int | None = Q8_BLOCK):
    """K: float16 [..., d].  Returns (codes int8 [..., d], scales float16 [..., d/block],
    pre float32 [..., d]) where pre = k * (1/s) is the value that was rounded.

    Per block:  amax = max|k|;  s = fp16(min(fp32(amax) / 127, 65504))  (stored; the minimum only acts
    on bfloat16 inputs beyond 8.3e6, which then saturate);  codes are formed with the
    STORED scale, inv = fp32(1)/fp32(s), q = clip(rint(fp32(k) * inv), -128, 127), ties to even;
    an all-zero block stores s = 0 and zero codes.  ``block=None``: one block = the whole tensor.
    """
    K = _as_f32_input(K, "K")
    d = K.shape[-1]
    if block is None:
        kb = K.reshape(1, -1)
    else:
        if d % block:
            raise ValueError("head_dim must be a multiple of the block size")
        kb = K.reshape(K.shape[:-1] + (d // block, block))
    k32 = kb.astype(np.float32)
    amax = np.max(np.abs(k32), axis=-1)
    s16 = np.minimum((amax / np.float32(127.0)).astype(np.float32), np.float32(FP16_MAX)).astype(np.float16)
    s32 = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(s32 > 0, np.float32(1.0) / s32, np.float32(0.0)).astype(np.float32)
    pre = (k32 * inv[..., None]).astype(np.float32)
    q = np.clip(np.rint(pre), -128, 127).astype(np.int8)
    if block is None:
        return q.reshape(K.shape), s16.reshape(()), pre.reshape(K.shape)
    return q.reshape(K.shape), s16, pre.reshape(K.shape)


def k_decode(codes, scales, block: int | None = Q8_BLOCK):
    """K_dequant = Kq * s  (float64 holds the fp32 product exactly)."""
    codes = np.asarray(codes)
    s = np.asarray(scales).astype(np.float64)
    if block is None:
        return codes.astype(np.float64) * s
    d = codes.shape[-1]
    q = codes.reshape(codes.shape[:-1] + (d // block, block)).astype(np.float64)
    return (q * s[..., None]).reshape(codes.shape)


# --------------------------------------------------------------------------- #
# Values: FWHT rotation + 3-bit Lloyd-Max
# --------------------------------------------------------------------------- #
def v_rotate(V, signs=None):
    """V_rot = FWHT(V)/sqrt(d) along head_dim (step 1 of the value quantizer); with a sign diagonal
    (rotation_signs) V_rot = FWHT(D V)/sqrt(d)."""
    V = np.asarray(V)
    d = V.shape[-1]
    v = V.astype(np.float64)
    if signs is not None:
        v = v * signs
    return fwht(v) / math.sqrt(d)


def v_quantize(v_rot, bits: int = V_BITS):
    """Nearest-centroid index; a tie goes to the lower index, i.e. idx = #{k : v_rot > t_k}
    (step 2 of the value quantizer)."""
    _, t = codebook(bits)
    idx = np.zeros(np.shape(v_rot), dtype=np.uint8)
    for tk in t:
        idx += (v_rot > tk).astype(np.uint8)
    return idx


def v_encode(V, signs=None, bits: int = V_BITS):
    """V: float16 [..., d] -> (idx uint8 [..., d] in 0..2^bits-1, v_rot float64 [..., d])."""
    V = _as_f32_input(V, "V")
    v_rot = v_rotate(V, signs)
    return v_quantize(v_rot, bits), v_rot


def v_pack(idx, bits: int = V_BITS):
    """Canonical bit-packing: code j occupies stream bits b*j..b*j+b-1 (LSB first); stream bit i is
    bit (i mod 8) of byte floor(i/8).  [..., d] -> uint8 [..., b*d/8]."""
    idx = np.asarray(idx, dtype=np.uint8)
    d = idx.shape[-1]
    if (d * bits) % 8:
        raise ValueError("bits*d must be a multiple of 8")
    stream = ((idx[..., :, None] >> np.arange(bits, dtype=np.uint8)) & 1).astype(np.uint8)
    stream = stream.reshape(idx.shape[:-1] + (d * bits,))
    return np.packbits(stream, axis=-1, bitorder="little")


def v_unpack(packed, d: int, bits: int = V_BITS):
    packed = np.asarray(packed, dtype=np.uint8)
    stream = np.unpackbits(packed, axis=-1, bitorder="little")[..., : d * bits]
    stream = stream.reshape(packed.shape[:-1] + (d, bits)).astype(np.uint8)
    return (stream << np.arange(bits, dtype=np.uint8)).sum(axis=-1).astype(np.uint8)


def v_decode(idx, signs=None, bits: int = V_BITS):
    """V_dequant = H c[idx] / sqrt(d)  (true inverse of the normalized rotation); with a sign diagonal
    D H c[idx] / sqrt(d), the inverse of H D / sqrt(d)."""
    c, _ = codebook(bits)
    idx = np.asarray(idx)
    d = idx.shape[-1]
    v = fwht(c[idx]) / math.sqrt(d)
    return v if signs is None else v * signs


# --------------------------------------------------------------------------- #
# Values, variant with a per-vector scale
# --------------------------------------------------------------------------- #
V_SCALE_MAX = 128.0    # largest stored scale (a format limit: probability x scale must fit fp16)


def v_scale(V):
    """Per-vector scale of the scaled-values variant.  Returns (g16 float16 [...], rms float64 [...]).

    rms = ||v||_2 / sqrt(d).  The rotation is orthonormal, so this is also the root mean square of the
    rotated coordinates; dividing by it gives the unit-variance coordinates that the N(0,1) codebook
    is optimal for (section "TurboQuant": unit-norm input, coordinates ~ N(0, 1/d), i.e. the same
    thing up to the factor sqrt(d) that the codebook's own scaling absorbs).  Stored value:
    g = fp16(min(rms, V_SCALE_MAX)), rounded once, to nearest even."""
    v = np.asarray(V).astype(np.float64)
    rms = np.sqrt(np.mean(v * v, axis=-1))
    return np.minimum(rms, V_SCALE_MAX).astype(np.float16), rms


def v_quantize_scaled(v_rot, g16, bits: int = V_BITS):
    """idx = #{k : v_rot > t_k * g}: the quantizer of v_quantize applied to v_rot / g, written without
    the division.  A vector whose scale is stored as zero decodes to the zero vector whatever its
    codes; it gets the codes of the zero vector, 2^(bits-1) - 1 (as v_quantize gives for 0; 3 at 3 bits)."""
    _, t = codebook(bits)
    g = np.asarray(g16).astype(np.float64)[..., None]
    idx = np.zeros(np.shape(v_rot), dtype=np.uint8)
    for tk in t:
        idx += (v_rot > tk * g).astype(np.uint8)
    return np.where(g > 0, idx, np.uint8((1 << bits) // 2 - 1)).astype(np.uint8)


def v_encode_scaled(V, signs=None, bits: int = V_BITS):
    """V: float16 [..., d] -> (idx uint8 [..., d], g16 float16 [...], v_rot float64 [..., d],
    rms float64 [...])."""
    V = _as_f32_input(V, "V")
    g16, rms = v_scale(V)
    v_rot = v_rotate(V, signs)
    return v_quantize_scaled(v_rot, g16, bits), g16, v_rot, rms


def v_decode_scaled(idx, g16, signs=None, bits: int = V_BITS):
    """V_dequant = g * H c[idx] / sqrt(d)  (g * D H c[idx] / sqrt(d) with a sign diagonal)."""
    return v_decode(idx, signs, bits) * np.asarray(g16).astype(np.float64)[..., None]


# --------------------------------------------------------------------------- #
# Values, variant: uniform int8 without rotation (the paper's proposed ablation)
# --------------------------------------------------------------------------- #
def v_encode_int8(V):
    """V: float16 [..., d] -> (codes int8 [..., d], scales float16 [...], pre float32 [..., d]).

    The key quantizer's formula (section "Compression Scheme", key quantization) on each value vector,
    one scale per vector: s = fp16(min(fp32(max|v|) / 127, V_SCALE_MAX)) (stored), codes formed with the
    stored scale, inv = fp32(1)/fp32(s), q = clip(rint(fp32(v) * inv), -128, 127), ties to even; a zero
    vector stores s = 0 and zero codes.  The cap is the same format limit as for the scaled variant:
    only with max|v| > 127 * 128 does the clip act, and elements beyond the range saturate at code
    127 or -128."""
    v32 = _as_f32_input(V, "V")
    amax = np.max(np.abs(v32), axis=-1)
    s16 = np.minimum((amax / np.float32(127.0)).astype(np.float32), np.float32(V_SCALE_MAX)).astype(np.float16)
    s32 = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(s32 > 0, np.float32(1.0) / s32, np.float32(0.0)).astype(np.float32)
    pre = (v32 * inv[..., None]).astype(np.float32)
    q = np.clip(np.rint(pre), -128, 127).astype(np.int8)
    return q, s16, pre


def v_decode_int8(codes, scales):
    """V_dequant = q * s."""
    return np.asarray(codes).astype(np.float64) * np.asarray(scales).astype(np.float64)[..., None]


# --------------------------------------------------------------------------- #
# Pool = encode of a whole [L, H, T, d] cache; decode back
# --------------------------------------------------------------------------- #
def pool_encode(K, V, scaled_values: bool = False, int8_values: bool = False, sign_seed: int = 0,
                key_per_tensor: bool = False, value_bits: int = V_BITS):
    """K, V float16 [L, H, T, d] -> dict with the canonical stored arrays and the pre-rounding
    values a parity test needs to find elements that sit on a decision threshold.  sign_seed != 0: the
    rotation carries the sign diagonal rotation_signs(sign_seed, d) (not with int8 values, which are
    not rotated).  key_per_tensor: one key scale per layer tensor [H, T, d], s = max|K|/127 over the
    whole tensor -- the key formula exactly as section "Compression Scheme" prints it -- instead of one
    per block of 32; k_scales is then float16 [L].  value_bits: bits per value code (the paper's 3, or 2 or 4
    with the Lloyd-Max codebook of that size)."""
    if key_per_tensor:
        K = np.asarray(K)
        per_layer = [k_encode(K[l], block=None) for l in range(K.shape[0])]
        k_codes = np.stack([p[0] for p in per_layer])
        k_scales = np.array([p[1] for p in per_layer], dtype=np.float16)
        k_pre = np.stack([p[2] for p in per_layer])
    else:
        k_codes, k_scales, k_pre = k_encode(K)
    out = {"k_codes": k_codes, "k_scales": k_scales, "k_pre": k_pre}
    if int8_values:
        if sign_seed:
            raise ValueError("int8 values are not rotated")
        v_codes, v_scales, v_pre = v_encode_int8(V)
        out.update(v_codes=v_codes, v_scales=v_scales, v_pre=v_pre)
        return out
    signs = rotation_signs(sign_seed, np.shape(V)[-1]) if sign_seed else None
    if scaled_values:
        v_idx, g16, v_rot, rms = v_encode_scaled(V, signs, value_bits)
        out.update(v_scales=g16, v_rms=rms)
    else:
        v_idx, v_rot = v_encode(V, signs, value_bits)
    out.update(v_packed=v_pack(v_idx, value_bits), v_idx=v_idx, v_rot=v_rot, v_bits=value_bits)
    if signs is not None:
        out["v_signs"] = signs
    return out


def pool_decode(pool):
    if pool["k_scales"].ndim == 1:      # one scale per layer tensor
        K_hat = np.stack([k_decode(pool["k_codes"][l], pool["k_scales"][l], block=None)
                          for l in range(pool["k_codes"].shape[0])])
    else:
        K_hat = k_decode(pool["k_codes"], pool["k_scales"])
    if "v_codes" in pool:
        return K_hat, v_decode_int8(pool["v_codes"], pool["v_scales"])
    d = pool["k_codes"].shape[-1]
    bits = pool.get("v_bits", V_BITS)
    idx = v_unpack(pool["v_packed"], d, bits)
    signs = pool.get("v_signs")
    V_hat = v_decode_scaled(idx, pool["v_scales"], signs, bits) if "v_scales" in pool else v_decode(idx, signs, bits)
    return K_hat, V_hat


def stored_bytes(L: int, H: int, T: int, d: int, scaled_values: bool = False, int8_values: bool = False,
                 key_per_tensor: bool = False, value_bits: int = V_BITS) -> dict:
    """Byte accounting (section "Compression Scheme", paragraph "Compression ratio")."""
    n = L * H * T
    k_codes = n * d
    k_scales = L * 2 if key_per_tensor else n * (d // Q8_BLOCK) * 2
    v_codes = n * d if int8_values else n * d * value_bits // 8
    v_scales = n * 2 if (scaled_values or int8_values) else 0
    dense16 = 2 * n * d * 2
    packed = k_codes + k_scales + v_codes + v_scales
    return {
        "k_codes": k_codes, "k_scales": k_scales, "v_codes": v_codes, "v_scales": v_scales, "packed": packed,
        "dense16": dense16,
        "ratio_payload": 16.0 / ((8 + V_BITS) / 2.0),      # the paper's 16/5.5
        "ratio_stored": dense16 / packed,                   # with the fp16 block scales
    }


# --------------------------------------------------------------------------- #
# Read path: N agents' decode attention over the shared pool
# --------------------------------------------------------------------------- #
def keys_as_fp16(K_hat):
    """The decoded keys as the paper's read path holds them: section "DynamicCache Injection" casts the
    decompressed tensors to the model's 16-bit dtype before they enter an agent's cache, so attention there runs
    over K rounded once (to nearest, ties to even) to that type.  Reading taken for the optional reduced key
    precision of the attention call: fp16, the 16-bit type of this build's dense tensors.  Returns float64."""
    return np.asarray(K_hat, dtype=np.float64).astype(np.float16).astype(np.float64)


def softmax_attend_one(q, Kmat, Vmat, scale):
    """One query vector against T keys/values, float64: the textbook definition."""
    s = (Kmat @ q) * scale
    s = s - np.max(s)
    p = np.exp(s)
    p /= np.sum(p)
    return p @ Vmat


def pool_attend(K_hat, V_hat, Q, scale: float | None = None, tails=None, tail_causal: bool = False):
    """K_hat, V_hat: decoded pool, float64 [L, H, T, d].
    Q: [L, A, nq, q_heads, d] (any float dtype); q head h reads kv head h // (q_heads // H).
    tails: optional list over agents of (tail_K, tail_V) float16 [L, H, t_a, d] (t_a may be 0) or
    None: the agent's private, uncompressed continuation, attended together with the pool.
    No mask by default: each query sees the whole pool and its agent's whole tail.  With
    tail_causal the agent's nq queries are taken to sit at its last nq tail positions (a multi-token
    decode step): query i sees the pool and the first t_a - (nq - 1 - i) tail tokens, i.e. the last
    query sees everything and each earlier one a token less (ordinary causal attention among them).
    Returns float64 [L, A, nq, q_heads, d]."""
    K_hat = np.asarray(K_hat, dtype=np.float64)
    V_hat = np.asarray(V_hat, dtype=np.float64)
    Q = np.asarray(Q).astype(np.float64)
    L, H, T, d = K_hat.shape
    Lq, A, nq, q_heads, dq = Q.shape
    if (Lq, dq) != (L, d) or q_heads % H:
        raise ValueError("shape mismatch")
    G = q_heads // H
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros_like(Q)
    for l in range(L):
        for a in range(A):
            tail = None if tails is None else tails[a]
            for h in range(q_heads):
                kv = h // G
                for i in range(nq):
                    Km, Vm = K_hat[l, kv], V_hat[l, kv]
                    if tail is not None:
                        t_a = tail[0].shape[2]
                        seen = max(0, t_a - (nq - 1 - i)) if tail_causal else t_a
                        if seen > 0:
                            Km = np.concatenate([Km, np.asarray(tail[0][l, kv, :seen], dtype=np.float64)], axis=0)
                            Vm = np.concatenate([Vm, np.asarray(tail[1][l, kv, :seen], dtype=np.float64)], axis=0)
                    out[l, a, i, h] = softmax_attend_one(Q[l, a, i, h], Km, Vm, scale)
    return out
