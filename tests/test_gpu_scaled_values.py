"""GPU parity tests of the scaled-values codec (a per-vector fp16 scale next to the 3-bit codes): the
HIP path through the C ABI against the CPU oracle's scaled variant on identical seeded inputs."""
import math

import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu


def _wide_values(rng, shape, sigma=1.0):
    """Value vectors whose lengths spread over more than an order of magnitude."""
    scale = np.exp(sigma * rng.standard_normal(shape[:-1] + (1,)))
    return (rng.standard_normal(shape) * scale).astype(np.float16)


@pytest.fixture(scope="module")
def tiny_s():
    cfg = W.CONFIGS[1]
    K, V = W.kv_pool(cfg)
    rng = np.random.default_rng(3)
    return Case(cfg, K, _wide_values(rng, V.shape), scaled_values=True)


@pytest.fixture(scope="module")
def llama_s():
    cfg = W.CONFIGS[3].scaled(layers=2, tokens=1500)
    K, V = W.kv_pool(cfg)
    rng = np.random.default_rng(4)
    return Case(cfg, K, _wide_values(rng, V.shape), scaled_values=True)


@pytest.mark.parametrize("name", ["tiny_s", "llama_s"])
def test_scaled_encode_bit_exact_and_decode_within_tolerance(name, request):
    case = request.getfixturevalue(name)
    pu = _pu()
    n = case.K.size
    assert case.k_mis <= 1e-5 * n and case.v_mis <= 1e-4 * n
    pu.compare_decode(case.pool, case.ref, case.dirty)
    cfg = case.cfg
    b = O.stored_bytes(cfg.layers, cfg.kv_heads, 32 * math.ceil(cfg.tokens / 32), cfg.head_dim, scaled_values=True)
    assert case.pool.nbytes == b["packed"]
    # the variant does what it is for: on vectors of very different lengths the relative error is the
    # codebook's own (about 0.035), which the unscaled codec misses by far
    V64 = case.V.astype(np.float64)
    _, Vg = case.pool.decode(torch.float32)
    rel = ((Vg.cpu().numpy() - V64) ** 2).sum(-1) / np.maximum((V64 ** 2).sum(-1), 1e-30)
    assert 0.03 < rel.mean() < 0.04
    plain = _pu().gpu_pool(case.K, case.V)
    _, Vp = plain.decode(torch.float32)
    rel_p = ((Vp.cpu().numpy() - V64) ** 2).sum(-1) / np.maximum((V64 ** 2).sum(-1), 1e-30)
    assert rel_p.mean() > 3 * rel.mean()


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("T", [1, 33, 95, 257])
def test_scaled_ragged_token_counts(d, T):
    pu = _pu()
    rng = np.random.default_rng(200 * d + T)
    K = (rng.standard_normal((2, 3, T, d)) * np.exp(rng.standard_normal((2, 3, T, 1)))).astype(np.float16)
    V = _wide_values(rng, (2, 3, T, d))
    case = Case(W.PoolConfig(0, "ragged", 2, 3, 6, d, T, 2, 1), K, V, scaled_values=True)
    pu.compare_decode(case.pool, case.ref, case.dirty)
    Q = rng.standard_normal((2, 2, 1, 6, d)).astype(np.float16)
    pk = _pk()
    case.attend_check(Q)
    case.attend_check(Q, kernel=pk.KERNEL_VECTOR)


def test_scaled_degenerate_vectors():
    pu = _pu()
    d, T = 128, 40
    rng = np.random.default_rng(9)
    K = rng.standard_normal((1, 2, T, d)).astype(np.float16)
    V = np.zeros((1, 2, T, d), dtype=np.float16)          # zero vectors: scale 0, codes 3
    V[0, 0, 2] = 0.25                                     # constant: spike at rotated coordinate 0
    V[0, 0, 3, 17] = 8.0                                  # spike: +-1 in units of the scale everywhere
    V[0, 1, 9] = 300.0                                    # rms above the format limit: scale 128
    V[0, 1, 10] = (rng.standard_normal(d) * 400.0).astype(np.float16)
    V[0, 1, 11, 5] = 6e-8                                 # too short for an fp16 scale: stored as zero
    V[0, 1, 12] = (rng.standard_normal(d) * 3e-6).astype(np.float16)   # subnormal fp16 scale
    V[0, 1, 13] = (rng.standard_normal(d) * 1e-3).astype(np.float16)
    case = Case(W.PoolConfig(0, "degenerate", 1, 2, 2, d, T, 1, 1), K, V, scaled_values=True)
    assert case.v_mis == 0
    pu.compare_decode(case.pool, case.ref, case.dirty)
    gs = case.pool.export_value_scales().cpu().numpy()
    assert gs[0, 0, 0] == 0 and gs[0, 1, 11] == 0 and gs[0, 0, 2] == np.float16(0.25)
    assert gs[0, 1, 9] == np.float16(128.0) and gs[0, 1, 10] == np.float16(128.0)
    assert 0 < gs[0, 1, 12] < 6.2e-5                      # a subnormal fp16
    vp = case.pool.export()[2].cpu().numpy()
    assert np.all(O.v_unpack(vp, d)[0, 1, 11] == 3)
    Q = rng.standard_normal((1, 1, 1, 2, d)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, kernel=_pk().KERNEL_VECTOR)


def test_scaled_attend_llama_shape_all_kernels_and_splits(llama_s):
    pk = _pk()
    cfg = llama_s.cfg
    Q = W.queries(cfg)                                    # 15 agents x 4 heads per KV head: 60 rows, two row tiles
    llama_s.attend_check(Q)
    llama_s.attend_check(Q, splits=1)                     # fused epilogue, no merge kernel
    llama_s.attend_check(Q, splits=5)
    llama_s.attend_check(Q[:1], layer_begin=0, layer_end=1, kernel=pk.KERNEL_VECTOR)
    llama_s.attend_check(Q[:, :3])                        # 12 rows: one row tile
    llama_s.attend_check(Q[:, :3], splits=1)
    llama_s.attend_check(Q[1:], layer_begin=1, layer_end=2, scale=0.05)


def test_scaled_attend_tiny_d64_with_tails(tiny_s):
    cfg = tiny_s.cfg
    tails = W.tails(cfg, [70, 70, 70])
    tiny_s.attend_check(W.queries(cfg, step=2), tails_np=tails, tails_len=[70, 0, 13])
    tiny_s.attend_check(W.queries(cfg))
    tiny_s.attend_check(W.queries(cfg), kernel=_pk().KERNEL_VECTOR)


def test_scaled_attend_with_private_tails(llama_s):
    cfg = llama_s.cfg
    lens = [0, 1, 5, 63, 64, 17, 0, 2, 33, 64, 9, 40, 1, 64, 3][: cfg.agents]
    tails = W.tails(cfg.scaled(cid=4), [64] * cfg.agents)
    llama_s.attend_check(W.queries(cfg, step=1), tails_np=tails, tails_len=lens)


def test_scaled_attend_result_does_not_depend_on_other_agents(llama_s):
    pu = _pu()
    Q = W.queries(llama_s.cfg)
    full = llama_s.pool.attend(pu.dev(Q))
    part = llama_s.pool.attend(pu.dev(Q[:, [0, 7, 14]]))
    assert torch.equal(part, full[:, [0, 7, 14]])


def test_scaled_large_scales_times_large_probabilities_stay_finite():
    # the P.V operand is probability x scale in fp16: the largest scale (128) with scores that climb just
    # slowly enough that the softmax reference is never raised (probabilities up to 2^8) must not overflow
    pu = _pu()
    rng = np.random.default_rng(13)
    d, T = 128, 320
    q = rng.standard_normal(d).astype(np.float32)
    q /= np.linalg.norm(q)
    # natural-log units, e^5.5 = 2^7.9; the first tile is flat at 0 and fixes the reference there
    ramp = np.concatenate([np.zeros(32), np.linspace(0.0, 5.5, T - 32)])[:, None]
    K = (ramp * q[None, :]).astype(np.float16)[None, None]
    V = (rng.standard_normal((1, 1, T, d)) * 300.0).astype(np.float16)
    case = Case(W.PoolConfig(0, "ramp", 1, 1, 1, d, T, 1, 1), K, V, scaled_values=True)
    assert float(case.ref["v_scales"].min()) == 128.0
    Q = np.broadcast_to(q.astype(np.float16), (1, 1, 1, 1, d)).copy()
    Kh, Vh = case.decoded()
    ref = O.pool_attend(Kh, Vh, Q, scale=1.0)
    for splits in (1, 2):
        out = case.pool.attend(pu.dev(Q), scale=1.0, splits=splits)
        torch.cuda.synchronize()
        g = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all()
        assert np.all(np.abs(g - ref) <= pu.attend_row_atol(Kh, Vh, Q, scale=1.0))   # values are ~128 x N(0, 1)


@pytest.mark.parametrize("d,chunks", [(128, [37, 1, 90, 32, 5]), (64, [1, 30, 33, 95])])
def test_scaled_append_in_chunks_equals_one_encode(d, chunks):
    pk = _pk()
    pu = _pu()
    rng = np.random.default_rng(11 * d + len(chunks))
    Lr, H, cap = 2, 3, sum(chunks) + 40
    T = sum(chunks)
    K = (rng.standard_normal((Lr, H, T, d)) * np.exp(0.7 * rng.standard_normal((Lr, H, T, 1)))).astype(np.float16)
    V = _wide_values(rng, (Lr, H, T, d))
    pool = pk.Pool(Lr, H, d, cap, value_codec=pk.VALUES_TQ3_SCALED).bind()
    pool.storage.fill_(0xA5)
    Q = rng.standard_normal((Lr, 3, 1, 2 * H, d)).astype(np.float16)
    pos = 0
    for n in chunks:
        pool.append(pu.dev(np.ascontiguousarray(K[:, :, pos:pos + n])), pu.dev(np.ascontiguousarray(V[:, :, pos:pos + n])))
        pos += n
        ref = O.pool_encode(K[:, :, :pos], V[:, :, :pos], scaled_values=True)
        dirty, _, _ = pu.compare_codes(pool, ref)
        pu.compare_decode(pool, ref, dirty)
        Kh, Vh = O.pool_decode(ref)
        out = pool.attend(pu.dev(Q))
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0, atol=pu.attend_row_atol(Kh, Vh, Q))


def test_value_scale_export_is_refused_for_the_papers_codec():
    pk = _pk()
    pu = _pu()
    K, V = W.kv_pool(W.CONFIGS[1])
    pool = pu.gpu_pool(K, V)
    with pytest.raises(pk.PolyKVError) as e:
        pool.export_value_scales()
    assert e.value.status == pk.ESTATE
