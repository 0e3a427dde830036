"""GPU parity tests at head_dim 256: the HIP path through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu


def _arrays(L, H, T, d, seed, value_sigma=0.3):
    rng = np.random.default_rng(seed)
    K = (rng.standard_normal((L, H, T, d)) * np.exp(0.5 * rng.standard_normal((L, H, 1, d)))).astype(np.float16)
    V = (rng.standard_normal((L, H, T, d)) * np.exp(value_sigma * rng.standard_normal((L, H, T, 1)))).astype(np.float16)
    return K, V


@pytest.mark.parametrize("codec", ["tq3", "scaled", "int8"])
@pytest.mark.parametrize("T", [1, 95, 700])
def test_d256_encode_decode_attend(codec, T):
    pu, pk = _pu(), _pk()
    L, H, d, A, qh = 2, 2, 256, 5, 8
    K, V = _arrays(L, H, T, d, 7 * T + len(codec), 0.3 if codec == "tq3" else 1.0)
    cfg = W.PoolConfig(0, "d256", L, H, qh, d, T, A, 1)
    case = Case(cfg, K, V, scaled_values=codec == "scaled", int8_values=codec == "int8")
    n = K.size
    assert case.k_mis <= 1e-5 * n + 1 and case.v_mis <= 1e-4 * n + 1
    pu.compare_decode(case.pool, case.ref, case.dirty)
    b = O.stored_bytes(L, H, 32 * ((T + 31) // 32), d, scaled_values=codec == "scaled", int8_values=codec == "int8")
    assert case.pool.nbytes == b["packed"]
    rng = np.random.default_rng(T)
    Q = rng.standard_normal((L, A, 1, qh, d)).astype(np.float16)       # 20 rows per KV head
    case.attend_check(Q)
    case.attend_check(Q, splits=1)
    if T <= 95:
        case.attend_check(Q, kernel=pk.KERNEL_VECTOR)
    tails = [(rng.standard_normal((L, H, 40, d)).astype(np.float16), rng.standard_normal((L, H, 40, d)).astype(np.float16))
             for _ in range(A)]
    case.attend_check(Q, tails_np=tails, tails_len=[0, 1, 40, 17, 33])


def test_d256_many_rows_sign_diagonal_bf16_and_append():
    pu, pk = _pu(), _pk()
    L, H, d, T, A, qh = 1, 2, 256, 300, 12, 16                          # 96 rows per KV head: three row blocks
    K, V = _arrays(L, H, T, d, 99)
    Kb, Vb = W.bf16_round(K.astype(np.float32)), W.bf16_round(V.astype(np.float32))
    seed = 424242
    ref = O.pool_encode(Kb, Vb, sign_seed=seed)
    pool = pk.Pool(L, H, d, T, sign_seed=seed).bind()
    pool.storage.fill_(0xA5)
    pool.append(pu.dev(Kb[:, :, :45], True), pu.dev(Vb[:, :, :45], True))
    pool.append(pu.dev(Kb[:, :, 45:], True), pu.dev(Vb[:, :, 45:], True))
    dirty, _, _ = pu.compare_codes(pool, ref)
    Kh, Vh = pu.compare_decode(pool, ref, dirty)
    rng = np.random.default_rng(1)
    Q = W.bf16_round(rng.standard_normal((L, A, 1, qh, d)).astype(np.float32))
    for splits in (0, 1):
        out = pool.attend(pu.dev(Q, True), splits=splits)
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0)
