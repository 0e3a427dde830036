"""The optional reduced key precision of pool_attend (POLYKV_KEY_PRECISION_FP16): scores over the dequantized keys
rounded once to fp16 -- what the paper's read path attends over after its cast to the model dtype (section
"DynamicCache Injection") -- against the oracle's attention over keys_as_fp16(K); the default stays exact."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import polykv as pk
from paper_2604_24971_amd import workloads as W
import parity_util as P

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,rows", [(128, 60), (64, 5), (128, 20)])
def test_fp16_keys_match_the_oracle_over_rounded_keys(d, rows):
    G = 4 if d == 128 else 1
    A = rows // G
    L, H, T = 2, 2, 777
    cfg = W.PoolConfig(31, "key-precision", L, H, H * G, d, T, A, 1)       # the outlier-channel distributions
    K, V = W.kv_pool(cfg)
    Q = W.queries(cfg)
    pool = P.gpu_pool(K, V)
    ref = O.pool_encode(K, V)
    P.compare_codes(pool, ref)
    Kh, Vh = O.pool_decode(ref)
    want16 = O.pool_attend(O.keys_as_fp16(Kh), Vh, Q)
    want = O.pool_attend(Kh, Vh, Q)
    for splits in (1, 0, 3):
        got16 = pool.attend(P.dev(Q), splits=splits, key_precision=pk.KEY_PRECISION_FP16)
        got = pool.attend(P.dev(Q), splits=splits)
        P.compare_attend(got16, want16, H)
        P.compare_attend(got, want, H)
        # the option really changes the scores: closer to its own oracle than to the other one
        e_own = np.abs(got16.cpu().numpy() - want16).max()
        assert np.abs(want16 - want).max() > 0
        assert e_own <= P.ATTEND_ATOL
    # the vector kernel and the other codecs ignore the option: exact keys
    got_v = pool.attend(P.dev(Q), kernel=pk.KERNEL_VECTOR, key_precision=pk.KEY_PRECISION_FP16)
    P.compare_attend(got_v, want, H)
    with pytest.raises(pk.PolyKVError):
        pool.attend(P.dev(Q), key_precision=7)
    with pytest.raises(pk.PolyKVError):
        pool.attend(P.dev(Q), scale=-1.0)
    with pytest.raises(pk.PolyKVError):
        pool.attend(P.dev(Q), scale=float("nan"))
    pool.close()
