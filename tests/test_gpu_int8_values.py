"""GPU parity tests of the int8 value codec (uniform int8 without rotation, one scale per vector -- the
ablation the paper proposes): the HIP path through the C ABI against the CPU oracle's variant."""
import math

import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu


def _values(rng, shape, sigma=1.0):
    scale = np.exp(sigma * rng.standard_normal(shape[:-1] + (1,)))
    return (rng.standard_normal(shape) * scale).astype(np.float16)


@pytest.fixture(scope="module")
def tiny_8():
    cfg = W.CONFIGS[1]
    K, V = W.kv_pool(cfg)
    return Case(cfg, K, _values(np.random.default_rng(5), V.shape), int8_values=True)


@pytest.fixture(scope="module")
def llama_8():
    cfg = W.CONFIGS[3].scaled(layers=2, tokens=1500)
    K, V = W.kv_pool(cfg)
    return Case(cfg, K, _values(np.random.default_rng(6), V.shape), int8_values=True)


@pytest.mark.parametrize("name", ["tiny_8", "llama_8"])
def test_int8_encode_bit_exact_and_decode_within_tolerance(name, request):
    case = request.getfixturevalue(name)
    pu = _pu()
    n = case.K.size
    assert case.k_mis <= 1e-5 * n and case.v_mis <= 1e-5 * n
    Kh, Vh = pu.compare_decode(case.pool, case.ref, case.dirty)
    cfg = case.cfg
    b = O.stored_bytes(cfg.layers, cfg.kv_heads, 32 * math.ceil(cfg.tokens / 32), cfg.head_dim, int8_values=True)
    assert case.pool.nbytes == b["packed"]
    # code * scale is exact in fp32: clean units decode bit for bit
    _, Vg = case.pool.decode(torch.float32)
    clean = ~case.dirty
    assert np.array_equal(Vg.cpu().numpy().astype(np.float64)[clean], Vh[clean])


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("T", [1, 33, 95, 257])
def test_int8_ragged_token_counts(d, T):
    pu = _pu()
    rng = np.random.default_rng(300 * d + T)
    K = (rng.standard_normal((2, 3, T, d)) * np.exp(rng.standard_normal((2, 3, T, 1)))).astype(np.float16)
    V = _values(rng, (2, 3, T, d))
    case = Case(W.PoolConfig(0, "ragged", 2, 3, 6, d, T, 2, 1), K, V, int8_values=True)
    pu.compare_decode(case.pool, case.ref, case.dirty)
    Q = rng.standard_normal((2, 2, 1, 6, d)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, kernel=_pk().KERNEL_VECTOR)


def test_int8_degenerate_vectors():
    pu = _pu()
    d, T = 128, 40
    rng = np.random.default_rng(19)
    K = rng.standard_normal((1, 2, T, d)).astype(np.float16)
    V = np.zeros((1, 2, T, d), dtype=np.float16)          # zero vectors: scale 0, codes 0
    V[0, 0, 2] = -0.375                                   # constant: every code -127
    V[0, 0, 3, 17] = 8.0                                  # spike
    V[0, 1, 9, :4] = [40000.0, -40000.0, 16256.0, 130.0]  # beyond the scale cap: saturates at 127 / -128
    V[0, 1, 11, 5] = 6e-8                                 # max/127 rounds to a zero scale
    V[0, 1, 12] = (rng.standard_normal(d) * 3e-4).astype(np.float16)   # subnormal fp16 scale
    V[0, 1, 13, :5] = [127.0, 0.5, 1.5, 2.5, -0.5]        # scale 1: exact ties, to even
    case = Case(W.PoolConfig(0, "degenerate", 1, 2, 2, d, T, 1, 1), K, V, int8_values=True)
    assert case.v_mis == 0
    pu.compare_decode(case.pool, case.ref, case.dirty)
    gs = case.pool.export_value_scales().cpu().numpy()
    vc = case.pool.export()[2].cpu().numpy()
    assert gs[0, 0, 0] == 0 and not vc[0, 0, 0].any()
    assert np.all(vc[0, 0, 2] == -127)
    assert gs[0, 1, 9] == np.float16(128.0) and vc[0, 1, 9, :4].tolist() == [127, -128, 127, 1]
    assert gs[0, 1, 11] == 0 and not vc[0, 1, 11].any()
    assert 0 < gs[0, 1, 12] < 6.2e-5
    assert vc[0, 1, 13, :5].tolist() == [127, 0, 2, 2, 0]
    Q = rng.standard_normal((1, 1, 1, 2, d)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, kernel=_pk().KERNEL_VECTOR)


def test_int8_attend_llama_shape_all_kernels_and_splits(llama_8):
    pk = _pk()
    cfg = llama_8.cfg
    Q = W.queries(cfg)
    llama_8.attend_check(Q)
    llama_8.attend_check(Q, splits=1)
    llama_8.attend_check(Q, splits=5)
    llama_8.attend_check(Q[:1], layer_begin=0, layer_end=1, kernel=pk.KERNEL_VECTOR)
    llama_8.attend_check(Q[:, :3])
    llama_8.attend_check(Q[:, :3], splits=1)
    llama_8.attend_check(Q[1:], layer_begin=1, layer_end=2, scale=0.05)


def test_int8_attend_with_private_tails(llama_8, tiny_8):
    cfg = llama_8.cfg
    lens = [0, 1, 5, 63, 64, 17, 0, 2, 33, 64, 9, 40, 1, 64, 3][: cfg.agents]
    tails = W.tails(cfg.scaled(cid=4), [64] * cfg.agents)
    llama_8.attend_check(W.queries(cfg, step=1), tails_np=tails, tails_len=lens)
    tcfg = tiny_8.cfg
    tiny_8.attend_check(W.queries(tcfg, step=2), tails_np=W.tails(tcfg, [70, 70, 70]), tails_len=[70, 0, 13])
    tiny_8.attend_check(W.queries(tcfg))
    tiny_8.attend_check(W.queries(tcfg), kernel=_pk().KERNEL_VECTOR)


def test_int8_attend_result_does_not_depend_on_other_agents(llama_8):
    pu = _pu()
    Q = W.queries(llama_8.cfg)
    full = llama_8.pool.attend(pu.dev(Q))
    part = llama_8.pool.attend(pu.dev(Q[:, [0, 7, 14]]))
    assert torch.equal(part, full[:, [0, 7, 14]])


@pytest.mark.parametrize("d,chunks", [(128, [37, 1, 90, 32, 5]), (64, [1, 30, 33, 95])])
def test_int8_append_in_chunks_equals_one_encode(d, chunks):
    pk = _pk()
    pu = _pu()
    rng = np.random.default_rng(13 * d + len(chunks))
    Lr, H, cap = 2, 3, sum(chunks) + 40
    T = sum(chunks)
    K = (rng.standard_normal((Lr, H, T, d)) * np.exp(0.7 * rng.standard_normal((Lr, H, T, 1)))).astype(np.float16)
    V = _values(rng, (Lr, H, T, d))
    pool = pk.Pool(Lr, H, d, cap, value_codec=pk.VALUES_INT8).bind()
    pool.storage.fill_(0xA5)
    Q = rng.standard_normal((Lr, 3, 1, 2 * H, d)).astype(np.float16)
    pos = 0
    for n in chunks:
        pool.append(pu.dev(np.ascontiguousarray(K[:, :, pos:pos + n])), pu.dev(np.ascontiguousarray(V[:, :, pos:pos + n])))
        pos += n
        ref = O.pool_encode(K[:, :, :pos], V[:, :, :pos], int8_values=True)
        dirty, _, _ = pu.compare_codes(pool, ref)
        pu.compare_decode(pool, ref, dirty)
        Kh, Vh = O.pool_decode(ref)
        out = pool.attend(pu.dev(Q))
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0, atol=pu.attend_row_atol(Kh, Vh, Q))
