"""Parity at full size and in the benchmark's launch configuration: the Llama-3-8B-shaped pool (32 layers x 8 KV
heads x head_dim 128 x 4096 tokens, 15 agents) and the SmolLM2-shaped pool (24 layers x 32 KV heads x head_dim 64
x 1851 tokens, 5 agents), all layers in one call -- exactly what bench.py times.  The oracle is run layer by
layer on the same seeded tensors; every layer, every KV head and every output row is compared."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W

pytestmark = pytest.mark.gpu


def _full_pool_against_oracle(cfg, value_codec=0, oracle_kw=None, attend_layers=None):
    """Encode, export, decode and attend the whole pool in single calls; compare every layer with the oracle.
    attend_layers: layers whose dequantization and attention are compared (default: all)."""
    import parity_util as pu
    from paper_2604_24971_amd import polykv as pk

    oracle_kw = oracle_kw or {}
    L, H, d, T = cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens
    K, V = W.kv_pool(cfg)
    Q = W.queries(cfg)
    pool = pk.Pool(L, H, d, T, value_codec=value_codec).bind()
    pool.encode(pu.dev(K), pu.dev(V))
    kc, ks, vp = (t.cpu().numpy() for t in pool.export())
    gs = pool.export_value_scales().cpu().numpy() if value_codec in (pk.VALUES_TQ3_SCALED, pk.VALUES_INT8) else None
    Kg, Vg = pool.decode(torch.float32)
    out = pool.attend(pu.dev(Q))                      # AUTO kernel, automatic splits: the bench path
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    wide_bar = value_codec != pk.VALUES_TQ3
    worst_att, mism_k, mism_v = 0.0, 0, 0
    for l in range(L):
        ref = O.pool_encode(K[l:l + 1], V[l:l + 1], **oracle_kw)
        # scales bit-exact, codes bit-exact except on a decision threshold, where the reference takes the
        # library's (neighbouring) code so that nothing below is masked
        mk, mv = pu.settle_codes(ref, kc[l:l + 1], ks[l:l + 1], vp[l:l + 1], None if gs is None else gs[l:l + 1])
        mism_k, mism_v = mism_k + mk, mism_v + mv
        if attend_layers is not None and l not in attend_layers:
            continue
        Kh, Vh = O.pool_decode(ref)
        for g, o in ((Kg[l].cpu().numpy(), Kh[0]), (Vg[l].cpu().numpy(), Vh[0])):   # 1e-3 relative, per vector
            err = np.abs(g - o).max(axis=-1)
            assert np.all(err <= pu.DEQUANT_RTOL * np.abs(o).max(axis=-1)), "layer %d dequantization" % l
        ref_out = O.pool_attend(Kh, Vh, Q[l:l + 1])[0]                        # [A, nq, q_heads, d]
        err = np.abs(out[l] - ref_out)
        bar = pu.attend_row_atol(Kh, Vh, Q[l:l + 1])[0] if wide_bar else pu.ATTEND_ATOL
        worst_att = max(worst_att, float(err.max()))
        assert np.all(err <= bar), "layer %d attention off by %g" % (l, err.max())
    n = K.size
    assert mism_k <= 1e-5 * n and mism_v <= 1e-4 * n
    print("full-size parity %s codec %d: worst attention error %.3g, threshold mismatches K %d V %d of %d" %
          (cfg.name, value_codec, worst_att, mism_k, mism_v, n))
    pool.close()


def test_llama_shape_full_pool_encode_decode_attend_against_oracle():
    _full_pool_against_oracle(W.CONFIGS[3])


def test_smollm2_shape_full_pool_encode_decode_attend_against_oracle():
    """Config 2 in full: 768 (layer, KV head) units, 5 query rows each."""
    _full_pool_against_oracle(W.CONFIGS[2])


def test_llama_shape_full_pool_scaled_values_codec_against_oracle():
    from paper_2604_24971_amd import polykv as pk
    _full_pool_against_oracle(W.CONFIGS[3], pk.VALUES_TQ3_SCALED, {"scaled_values": True}, attend_layers=range(1, 32, 8))


def test_llama_shape_full_pool_int8_values_codec_against_oracle():
    from paper_2604_24971_amd import polykv as pk
    _full_pool_against_oracle(W.CONFIGS[3], pk.VALUES_INT8, {"int8_values": True}, attend_layers=range(1, 32, 8))
