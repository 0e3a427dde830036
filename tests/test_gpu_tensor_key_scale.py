"""GPU parity tests of the key codec with one scale per layer tensor (the key formula exactly as the paper
prints it): the HIP path through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("codec", ["tq3", "scaled", "int8"])
@pytest.mark.parametrize("shape", ["tiny", "llama", "d256"])
def test_tensor_key_scale_encode_decode_attend(shape, codec):
    pu, pk = _pu(), _pk()
    if shape == "tiny":
        cfg = W.CONFIGS[1]
    elif shape == "llama":
        cfg = W.CONFIGS[3].scaled(layers=2, tokens=1100)
    else:
        cfg = W.PoolConfig(0, "d256", 2, 2, 8, 256, 333, 5, 1)
    K, V = W.kv_pool(cfg) if shape != "d256" else (None, None)
    if K is None:
        rng = np.random.default_rng(5)
        K = (rng.standard_normal((2, 2, 333, 256)) * np.array([1.0, 6.0])[:, None, None, None]).astype(np.float16)
        V = rng.standard_normal((2, 2, 333, 256)).astype(np.float16)
    case = Case(cfg, K, V, scaled_values=codec == "scaled", int8_values=codec == "int8", key_per_tensor=True)
    assert case.ref["k_scales"].shape == (cfg.layers,)
    n = K.size
    assert case.k_mis <= 1e-5 * n + 1 and case.v_mis <= 1e-4 * n + 1
    pu.compare_decode(case.pool, case.ref, case.dirty)
    # no per-block scales in the pool: head_dim/16 bytes less per vector, plus the layers' maxima
    blocked = O.stored_bytes(cfg.layers, cfg.kv_heads, 32 * ((cfg.tokens + 31) // 32), cfg.head_dim,
                             scaled_values=codec == "scaled", int8_values=codec == "int8")
    vectors = cfg.layers * cfg.kv_heads * 32 * ((cfg.tokens + 31) // 32)
    assert case.pool.nbytes == blocked["packed"] - vectors * cfg.head_dim // 16 + 256
    Q = W.queries(cfg) if shape != "d256" else np.random.default_rng(6).standard_normal((2, 5, 1, 8, 256)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, splits=1)
    if shape != "llama":
        case.attend_check(Q, kernel=pk.KERNEL_VECTOR)
    A = Q.shape[1]
    rng = np.random.default_rng(7)
    tails = [(rng.standard_normal((cfg.layers, cfg.kv_heads, 40, cfg.head_dim)).astype(np.float16),
              rng.standard_normal((cfg.layers, cfg.kv_heads, 40, cfg.head_dim)).astype(np.float16)) for _ in range(A)]
    case.attend_check(Q, tails_np=tails, tails_len=[(13 * a) % 41 for a in range(A)])
    if cfg.layers > 1:
        case.attend_check(Q[1:], layer_begin=1, layer_end=2)         # the second layer's own scale


def test_tensor_key_scale_zero_layer_reencode_and_no_append():
    pu, pk = _pu(), _pk()
    rng = np.random.default_rng(8)
    L, H, T, d = 2, 2, 70, 128
    K = rng.standard_normal((L, H, T, d)).astype(np.float16)
    K[1] = 0                                                       # an all-zero layer: scale 0, codes 0
    V = rng.standard_normal((L, H, T, d)).astype(np.float16)
    ref = O.pool_encode(K, V, key_per_tensor=True)
    pool = pk.Pool(L, H, d, T, key_codec=pk.KEYS_Q8_TENSOR).bind()
    pool.storage.fill_(0xA5)
    big = (K.astype(np.float32) * 50).astype(np.float16)
    pool.encode(pu.dev(big), pu.dev(V))                              # a first encode with larger keys ...
    pool.encode(pu.dev(K), pu.dev(V))                                # ... must not leave its maxima behind
    dirty, k_mis, _ = pu.compare_codes(pool, ref)
    assert k_mis == 0 and float(ref["k_scales"][1]) == 0.0
    Kh, Vh = pu.compare_decode(pool, ref, dirty)
    Q = rng.standard_normal((L, 3, 1, 4, d)).astype(np.float16)
    for splits in (0, 1):
        out = pool.attend(pu.dev(Q), splits=splits)
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0)
    with pytest.raises(pk.PolyKVError) as e:
        pool.append(pu.dev(K[:, :, :5]), pu.dev(V[:, :, :5]))
    assert e.value.status == pk.ESTATE
    # bfloat16 keys
    Kb = W.bf16_round(K.astype(np.float32) * 3)
    Vb = W.bf16_round(V.astype(np.float32))
    pool.encode(pu.dev(Kb, True), pu.dev(Vb, True))
    pu.compare_codes(pool, O.pool_encode(Kb, Vb, key_per_tensor=True))
