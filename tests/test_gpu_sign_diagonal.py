"""GPU parity tests of the rotation variant with a pseudorandom sign diagonal (v_rot = H D v / sqrt(d)):
the HIP path through the C ABI against the CPU oracle with the same seed."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu

SEED = 0x5EED5EED5EED


@pytest.mark.parametrize("scaled", [False, True])
@pytest.mark.parametrize("shape", ["tiny", "llama"])
def test_signed_rotation_encode_decode_attend(shape, scaled):
    pu, pk = _pu(), _pk()
    cfg = W.CONFIGS[1] if shape == "tiny" else W.CONFIGS[3].scaled(layers=2, tokens=1100)
    case = Case(cfg, scaled_values=scaled, sign_seed=SEED)
    assert "v_signs" in case.ref
    n = case.K.size
    assert case.k_mis <= 1e-5 * n and case.v_mis <= 1e-4 * n
    pu.compare_decode(case.pool, case.ref, case.dirty)
    # the diagonal matters: the same pool without it holds different codes
    plain = O.pool_encode(case.K, case.V, scaled_values=scaled)
    assert (plain["v_idx"] != case.ref["v_idx"]).mean() > 0.3
    Q = W.queries(cfg)
    case.attend_check(Q)                         # automatic splits (merge kernel)
    case.attend_check(Q, splits=1)               # fused epilogue
    case.attend_check(Q[:1], layer_begin=0, layer_end=1, kernel=pk.KERNEL_VECTOR)
    A = cfg.agents
    tails = W.tails(cfg.scaled(cid=4) if shape == "llama" else cfg, [40] * A)
    case.attend_check(W.queries(cfg, step=1), tails_np=tails, tails_len=[(11 * a) % 41 for a in range(A)])


def test_signed_rotation_on_structured_vectors_and_append():
    pu, pk = _pu(), _pk()
    rng = np.random.default_rng(3)
    L, H, T, d = 1, 2, 100, 128
    K = rng.standard_normal((L, H, T, d)).astype(np.float16)
    V = (1.0 + 0.05 * rng.standard_normal((L, H, T, d))).astype(np.float16)      # nearly constant vectors
    ref = O.pool_encode(K, V, sign_seed=SEED)
    pool = pk.Pool(L, H, d, T, sign_seed=SEED).bind()
    pool.storage.fill_(0xA5)
    pool.append(pu.dev(K[:, :, :37]), pu.dev(V[:, :, :37]))
    pool.append(pu.dev(K[:, :, 37:]), pu.dev(V[:, :, 37:]))
    dirty, _, _ = pu.compare_codes(pool, ref)
    Kh, Vh = pu.compare_decode(pool, ref, dirty)
    _, Vg = pool.decode(torch.float32)
    plain_pool = pu.gpu_pool(K, V)
    _, Vp = plain_pool.decode(torch.float32)
    V32 = torch.from_numpy(V.astype(np.float32)).cuda()
    assert float(((Vg - V32) ** 2).mean()) < 0.2 * float(((Vp - V32) ** 2).mean())
    with pytest.raises(pk.PolyKVError) as e:     # the diagonal is fixed once tokens are in
        _check_rc(pk, pool, 99)
    assert e.value.status == pk.ESTATE


def _check_rc(pk, pool, seed):
    pk._check(pk.lib.pool_set_sign_seed(pool._h, seed))
