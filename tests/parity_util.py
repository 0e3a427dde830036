"""Helpers for the GPU parity tests: run the same seeded tensors through the C-ABI library and the
CPU oracle and compare to the stated bars:
  * stored codes / scales bit-exact, except elements whose pre-rounding value (oracle's) lies within
    1e-6 of a decision threshold, which may take the neighbouring code;
  * dequantized K/V within 1e-3 relative, per vector, infinity norm;
  * attention output within 2e-3 absolute.
"""
import numpy as np
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import polykv as pk

CODE_WINDOW = 1e-6
DEQUANT_RTOL = 1e-3
ATTEND_ATOL = 2e-3


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def gpu_pool(K, V):
    L, H, T, d = K.shape
    pool = pk.Pool(L, H, d, T).bind()
    pool.storage.fill_(0xA5)            # stale bytes must never leak into results
    pool.encode(dev(K), dev(V))
    return pool


def compare_codes(pool, ref):
    """Returns a bool array [L, H] marking units where a (permitted) threshold mismatch occurred."""
    kc, ks, vp = (t.cpu().numpy() for t in pool.export())
    d = pool.head_dim
    # scales: bit-exact
    np.testing.assert_array_equal(ks.view(np.uint16), ref["k_scales"].view(np.uint16))
    # key codes
    k_diff = kc != ref["k_codes"]
    if k_diff.any():
        frac = np.abs(ref["k_pre"] - np.floor(ref["k_pre"]) - 0.5)
        assert np.all(frac[k_diff] <= CODE_WINDOW), "key code differs away from a rounding tie"
        assert np.all(np.abs(kc.astype(np.int32) - ref["k_codes"])[k_diff] == 1)
    # value codes
    v_idx = O.v_unpack(vp, d)
    v_diff = v_idx != ref["v_idx"]
    if v_diff.any():
        _, t = O.codebook()
        dist = np.min(np.abs(ref["v_rot"][v_diff][:, None] - t[None, :]), axis=1)
        assert np.all(dist <= CODE_WINDOW), "value code differs away from a threshold (max dist %g)" % dist.max()
        assert np.all(np.abs(v_idx.astype(np.int32) - ref["v_idx"])[v_diff] == 1)
    # packed stream identical wherever the codes are
    if not v_diff.any():
        np.testing.assert_array_equal(vp, ref["v_packed"])
    return k_diff.any(axis=(2, 3)) | v_diff.any(axis=(2, 3)), int(k_diff.sum()), int(v_diff.sum())


def compare_decode(pool, ref, dirty_units):
    Kh, Vh = O.pool_decode(ref)
    Kg, Vg = (t.cpu().numpy().astype(np.float64) for t in pool.decode(torch.float32))
    for name, g, o in (("K", Kg, Kh), ("V", Vg, Vh)):
        err = np.abs(g - o).max(axis=-1)
        bound = DEQUANT_RTOL * np.abs(o).max(axis=-1)
        bad = (err > bound) & ~dirty_units[:, :, None]
        assert not bad.any(), "%s dequant off by %g (bound %g)" % (name, err[bad].max(), bound[bad].min())
    # fp16 output = fp32 output rounded once
    Kg16, Vg16 = pool.decode(torch.float16)
    Kg32, Vg32 = pool.decode(torch.float32)
    assert torch.equal(Kg16, Kg32.to(torch.float16)) and torch.equal(Vg16, Vg32.to(torch.float16))
    return Kh, Vh


def compare_attend(out_gpu, out_ref, kv_heads, dirty_units=None, layer_begin=0, atol=ATTEND_ATOL):
    g = out_gpu.cpu().numpy().astype(np.float64)
    assert g.shape == out_ref.shape
    err = np.abs(g - out_ref)                       # [Ls, A, nq, q_heads, d]
    if dirty_units is not None and dirty_units.any():
        G = g.shape[3] // kv_heads
        mask = np.repeat(dirty_units[layer_begin:layer_begin + g.shape[0]], G, axis=1)   # [Ls, q_heads]
        err = np.where(mask[:, None, None, :, None], 0.0, err)
    assert np.isfinite(g).all()
    assert err.max() <= atol, "attention output off by %g" % err.max()
    return float(err.max())
