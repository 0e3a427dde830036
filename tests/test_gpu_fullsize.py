"""Parity at the benchmark's full size and launch configuration: the Llama-3-8B-shaped pool
(32 layers x 8 KV heads x head_dim 128 x 4096 tokens), 15 agents, all layers in one call -- exactly
what bench.py times.  The oracle is run layer by layer on the same seeded tensors."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_llama_shape_full_pool_encode_decode_attend_against_oracle():
    import parity_util as pu
    from paper_2604_24971_amd import polykv as pk

    cfg = W.CONFIGS[3]
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens
    K, V = W.kv_pool(cfg)
    Q = W.queries(cfg)
    pool = pk.Pool(L, H, d, T).bind()
    pool.encode(pu.dev(K), pu.dev(V))
    kc, ks, vp = (t.cpu().numpy() for t in pool.export())
    Kg, Vg = pool.decode(torch.float32)
    out = pool.attend(pu.dev(Q))                      # AUTO kernel, automatic splits: the bench path
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    _, thr = O.codebook()

    worst_att, mism_k, mism_v = 0.0, 0, 0
    for l in range(L):
        ref = O.pool_encode(K[l:l + 1], V[l:l + 1])
        # scales bit-exact, codes bit-exact except on a decision threshold
        assert np.array_equal(ks[l].view(np.uint16), ref["k_scales"][0].view(np.uint16)), "layer %d scales" % l
        kd = kc[l] != ref["k_codes"][0]
        if kd.any():
            frac = np.abs(ref["k_pre"][0] - np.floor(ref["k_pre"][0]) - 0.5)
            assert np.all(frac[kd] <= pu.CODE_WINDOW)
        v_idx = O.v_unpack(vp[l], d)
        vd = v_idx != ref["v_idx"][0]
        if vd.any():
            dist = np.min(np.abs(ref["v_rot"][0][vd][:, None] - thr[None, :]), axis=1)
            assert np.all(dist <= pu.CODE_WINDOW), "layer %d: value code off a threshold by %g" % (l, dist.max())
        mism_k += int(kd.sum())
        mism_v += int(vd.sum())
        dirty = kd.any(axis=(1, 2)) | vd.any(axis=(1, 2))                     # [H]
        if l % 4 != 1:          # codes and scales: every layer; dequantization and attention: every 4th
            continue
        # dequantized tensors within 1e-3 relative, per vector
        Kh, Vh = O.pool_decode(ref)
        for g, o in ((Kg[l].cpu().numpy(), Kh[0]), (Vg[l].cpu().numpy(), Vh[0])):
            err = np.abs(g - o).max(axis=-1)
            bound = pu.DEQUANT_RTOL * np.abs(o).max(axis=-1)
            assert not ((err > bound) & ~dirty[:, None]).any()
        # attention within 2e-3 absolute
        ref_out = O.pool_attend(Kh, Vh, Q[l:l + 1])[0]                        # [A, nq, q_heads, d]
        err = np.abs(out[l] - ref_out)
        mask = np.repeat(dirty, cfg.group)
        err[:, :, mask, :] = 0.0
        worst_att = max(worst_att, float(err.max()))
        assert err.max() <= pu.ATTEND_ATOL, "layer %d attention off by %g" % (l, err.max())
    n = K.size
    assert mism_k <= 1e-5 * n and mism_v <= 1e-4 * n
    print("full-size parity: worst attention error %.3g, threshold mismatches K %d V %d of %d" %
          (worst_att, mism_k, mism_v, n))


def test_llama_shape_full_pool_scaled_values_codec_against_oracle():
    """The same pool and launch configuration with the scaled-values codec; the oracle checks every
    eighth layer in full (scales, codes, dequantization, attention)."""
    import parity_util as pu
    from paper_2604_24971_amd import polykv as pk

    cfg = W.CONFIGS[3]
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens
    K, V = W.kv_pool(cfg)
    Q = W.queries(cfg)
    pool = pk.Pool(L, H, d, T, value_codec=pk.VALUES_TQ3_SCALED).bind()
    pool.encode(pu.dev(K), pu.dev(V))
    kc, ks, vp = (t.cpu().numpy() for t in pool.export())
    gs = pool.export_value_scales().cpu().numpy()
    Kg, Vg = pool.decode(torch.float32)
    out = pool.attend(pu.dev(Q))
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    _, thr = O.codebook()

    worst_att, mism_v, settled = 0.0, 0, 0
    for l in range(1, L, 8):
        ref = O.pool_encode(K[l:l + 1], V[l:l + 1], scaled_values=True)
        settled += pu.settle_value_scales(gs[l:l + 1], ref)
        assert np.array_equal(gs[l].view(np.uint16), ref["v_scales"][0].view(np.uint16))
        assert np.array_equal(ks[l].view(np.uint16), ref["k_scales"][0].view(np.uint16))
        v_idx = O.v_unpack(vp[l], d)
        vd = v_idx != ref["v_idx"][0]
        if vd.any():
            g = np.broadcast_to(ref["v_scales"][0].astype(np.float64)[..., None], v_idx.shape)[vd]
            dist = np.min(np.abs(ref["v_rot"][0][vd][:, None] - thr[None, :] * g[:, None]), axis=1) / g
            assert np.all(dist <= pu.CODE_WINDOW), "layer %d: value code off a threshold by %g" % (l, dist.max())
        mism_v += int(vd.sum())
        dirty = (kc[l] != ref["k_codes"][0]).any(axis=(1, 2)) | vd.any(axis=(1, 2))
        Kh, Vh = O.pool_decode(ref)
        o = Vh[0]
        err = np.abs(Vg[l].cpu().numpy() - o).max(axis=-1)
        assert not ((err > pu.DEQUANT_RTOL * np.abs(o).max(axis=-1)) & ~dirty[:, None]).any()
        ref_out = O.pool_attend(Kh, Vh, Q[l:l + 1])[0]
        err = np.abs(out[l] - ref_out)
        err[:, :, np.repeat(dirty, cfg.group), :] = 0.0
        worst_att = max(worst_att, float(err.max()))
        assert np.all(err <= pu.attend_row_atol(Kh, Vh, Q[l:l + 1])[0])
    print("full-size parity, scaled values: worst attention error %.3g, threshold mismatches V %d, "
          "scales settled at a rounding tie %d" % (worst_att, mism_v, settled))


def test_llama_shape_full_pool_int8_values_codec_against_oracle():
    """The same pool and launch configuration with the int8 value codec; the oracle checks every eighth
    layer in full (scales and codes bit-exact, dequantization exact, attention)."""
    import parity_util as pu
    from paper_2604_24971_amd import polykv as pk

    cfg = W.CONFIGS[3]
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens
    K, V = W.kv_pool(cfg)
    Q = W.queries(cfg)
    pool = pk.Pool(L, H, d, T, value_codec=pk.VALUES_INT8).bind()
    pool.encode(pu.dev(K), pu.dev(V))
    kc, ks, vc = (t.cpu().numpy() for t in pool.export())
    gs = pool.export_value_scales().cpu().numpy()
    Kg, Vg = pool.decode(torch.float32)
    out = pool.attend(pu.dev(Q))
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)

    worst_att, mism_v = 0.0, 0
    for l in range(1, L, 8):
        ref = O.pool_encode(K[l:l + 1], V[l:l + 1], int8_values=True)
        assert np.array_equal(gs[l].view(np.uint16), ref["v_scales"][0].view(np.uint16))
        vd = vc[l] != ref["v_codes"][0]
        if vd.any():
            frac = np.abs(ref["v_pre"][0] - np.floor(ref["v_pre"][0]) - 0.5)
            assert np.all(frac[vd] <= pu.CODE_WINDOW)
        mism_v += int(vd.sum())
        dirty = (kc[l] != ref["k_codes"][0]).any(axis=(1, 2)) | vd.any(axis=(1, 2))
        Kh, Vh = O.pool_decode(ref)
        assert np.array_equal(Vg[l].cpu().numpy().astype(np.float64)[~dirty], Vh[0][~dirty])   # code * s is exact
        ref_out = O.pool_attend(Kh, Vh, Q[l:l + 1])[0]
        err = np.abs(out[l] - ref_out)
        err[:, :, np.repeat(dirty, cfg.group), :] = 0.0
        worst_att = max(worst_att, float(err.max()))
        assert np.all(err <= pu.attend_row_atol(Kh, Vh, Q[l:l + 1])[0])
    print("full-size parity, int8 values: worst attention error %.3g, rounding-tie mismatches V %d" % (worst_att, mism_v))
