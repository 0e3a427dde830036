"""GPU parity tests of the value codec at 2 and 4 bits per coordinate (with and without the per-vector
scale): the HIP path through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu


def _values(rng, shape, sigma):
    return (rng.standard_normal(shape) * np.exp(sigma * rng.standard_normal(shape[:-1] + (1,)))).astype(np.float16)


@pytest.mark.parametrize("scaled", [False, True])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("shape", ["tiny", "llama", "d256"])
def test_value_bits_encode_decode_attend(shape, bits, scaled):
    pu, pk = _pu(), _pk()
    if shape == "tiny":
        cfg = W.CONFIGS[1]
    elif shape == "llama":
        cfg = W.CONFIGS[3].scaled(layers=2, tokens=1100)
    else:
        cfg = W.PoolConfig(0, "d256", 2, 2, 8, 256, 333, 5, 1)
    rng = np.random.default_rng(17 * bits + len(shape))
    L, H, T, d = cfg.layers, cfg.kv_heads, cfg.tokens, cfg.head_dim
    K = (rng.standard_normal((L, H, T, d)) * np.exp(0.5 * rng.standard_normal((L, H, 1, d)))).astype(np.float16)
    V = _values(rng, (L, H, T, d), 1.0 if scaled else 0.3)
    case = Case(cfg, K, V, scaled_values=scaled, value_bits=bits)
    n = K.size
    assert case.k_mis <= 1e-5 * n + 1 and case.v_mis <= 1e-4 * n + 1
    Kh, Vh = pu.compare_decode(case.pool, case.ref, case.dirty)
    b = O.stored_bytes(L, H, 32 * ((T + 31) // 32), d, scaled_values=scaled, value_bits=bits)
    assert case.pool.nbytes == b["packed"]
    # the codebook at work: relative error of the decoded values = its distortion (scaled codec, any length)
    if scaled:
        c, t = O.codebook(bits)
        V64 = V.astype(np.float64)
        rel = ((Vh - V64) ** 2).sum(-1) / np.maximum((V64 ** 2).sum(-1), 1e-30)
        assert abs(rel.mean() / O.lloyd_max_mse(c, t) - 1) < 0.05
    A, qh = cfg.agents, cfg.q_heads
    Q = rng.standard_normal((L, A, 1, qh, d)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, splits=1)
    if shape != "llama":
        case.attend_check(Q, kernel=pk.KERNEL_VECTOR)
    tails = [(rng.standard_normal((L, H, 40, d)).astype(np.float16), rng.standard_normal((L, H, 40, d)).astype(np.float16))
             for _ in range(A)]
    case.attend_check(Q, tails_np=tails, tails_len=[(13 * a) % 41 for a in range(A)])


@pytest.mark.parametrize("bits", [2, 4])
def test_value_bits_append_sign_diagonal_tensor_keys(bits):
    pu, pk = _pu(), _pk()
    rng = np.random.default_rng(5 + bits)
    L, H, T, d = 2, 3, 165, 128
    K = rng.standard_normal((L, H, T, d)).astype(np.float16)
    V = _values(rng, (L, H, T, d), 1.0)
    seed = 777
    codec = pu.value_codec_id(scaled_values=True, value_bits=bits)
    pool = pk.Pool(L, H, d, T + 40, value_codec=codec, sign_seed=seed).bind()
    pool.storage.fill_(0xA5)
    Q = rng.standard_normal((L, 3, 1, 6, d)).astype(np.float16)
    pos = 0
    for n in (37, 1, 90, 32, 5):
        pool.append(pu.dev(np.ascontiguousarray(K[:, :, pos:pos + n])), pu.dev(np.ascontiguousarray(V[:, :, pos:pos + n])))
        pos += n
        ref = O.pool_encode(K[:, :, :pos], V[:, :, :pos], scaled_values=True, sign_seed=seed, value_bits=bits)
        dirty, _, _ = pu.compare_codes(pool, ref)
        Kh, Vh = pu.compare_decode(pool, ref, dirty)
        out = pool.attend(pu.dev(Q))
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0, atol=pu.attend_row_atol(Kh, Vh, Q))
    # one key scale per layer tensor together with the other bit widths
    case = Case(W.PoolConfig(0, "kt", L, H, 6, d, T, 3, 1), K, V, value_bits=bits, key_per_tensor=True)
    pu.compare_decode(case.pool, case.ref, case.dirty)
    case.attend_check(Q)
    # degenerate vectors in the scaled codec: zero scale -> the code of zero everywhere
    Vz = np.zeros((1, 1, 40, d), dtype=np.float16)
    Vz[0, 0, 3] = 0.5
    Vz[0, 0, 4, 7] = 6e-8
    Kz = rng.standard_normal((1, 1, 40, d)).astype(np.float16)
    cz = Case(W.PoolConfig(0, "z", 1, 1, 1, d, 40, 1, 1), Kz, Vz, scaled_values=True, value_bits=bits)
    assert cz.v_mis == 0
    vp = cz.pool.export()[2].cpu().numpy()
    assert np.all(O.v_unpack(vp, d, bits)[0, 0, 4] == (1 << bits) // 2 - 1)
