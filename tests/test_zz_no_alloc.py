"""pool_attend_static, the entry point for callers that cannot allocate device memory, against pool_attend:
same kernels, same plan, so the outputs must be bit-identical -- on two calls in a row that share the
library's built-in scratch buffer, the second with a smaller input, with and without private tails."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_24971_amd import polykv as pk
from paper_2604_24971_amd import workloads as W

pytestmark = pytest.mark.gpu


def _raw_params(pool, Q, layer_begin, layer_end, splits, tails):
    p, keep = pool._params(Q, None, layer_begin, layer_end, None, tails, pk.KERNEL_AUTO, splits)
    return p, keep


def _both(pool, Q, layer_begin, layer_end, splits=0, tails=None):
    """One call through each entry point of the C ABI (raw ctypes, the binding only builds the struct)."""
    p, keep = _raw_params(pool, Q, layer_begin, layer_end, splits, tails)
    need = pk.lib.pool_attend_workspace(pool._h, C.byref(p))
    assert 0 < need <= pk.STATIC_WORKSPACE_BYTES
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    out_ref = torch.full(Q.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    out_st = torch.full(Q.shape, float("nan"), dtype=torch.float32, device="cuda:0")
    p.workspace_dev, p.workspace_bytes = ws.data_ptr(), need
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert pk.lib.pool_attend(pool._h, C.c_void_p(Q.data_ptr()), C.c_void_p(out_ref.data_ptr()), C.byref(p), stream) == pk.OK
    p.workspace_dev, p.workspace_bytes = None, 0          # ignored by the static entry point
    assert pk.lib.pool_attend_static(pool._h, C.c_void_p(Q.data_ptr()), C.c_void_p(out_st.data_ptr()), C.byref(p),
                                     stream) == pk.OK, pk.lib.polykv_last_error()
    torch.cuda.synchronize()
    assert torch.isfinite(out_ref).all()
    assert torch.equal(out_ref, out_st)
    return out_ref


def test_static_entry_point_matches_pool_attend_twice_in_a_row():
    from oracle import polykv_oracle as O
    L, H, d, T, A, qh = 2, 2, 128, 1000, 5, 8
    rng = np.random.default_rng(77)
    K = rng.standard_normal((L, H, T, d)).astype(np.float16)
    V = rng.standard_normal((L, H, T, d)).astype(np.float16)
    Q = rng.standard_normal((L, A, 1, qh, d)).astype(np.float16)
    pool = pk.Pool(L, H, d, T).bind()
    pool.encode(torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    Qd = torch.from_numpy(Q).cuda()
    # first call: both layers, split token range (partials go through the scratch buffer)
    out1 = _both(pool, Qd, 0, L, splits=4)
    # second call, smaller: one layer, fewer agents, other split count; stale partials of the first call remain
    Q2 = Qd[1:2, :2].contiguous()
    out2 = _both(pool, Q2, 1, 2, splits=3)
    # other split count: other softmax references, so other fp16 roundings of the probabilities
    assert torch.allclose(out2, out1[1:2, :2], atol=1e-3, rtol=0)
    # against the oracle, to the bar of the other parity tests
    ref = O.pool_encode(K, V)
    Kh, Vh = O.pool_decode(ref)
    want = O.pool_attend(Kh, Vh, Q)
    assert np.abs(out1.cpu().numpy() - want).max() <= 2e-3
    # third and fourth call with private tails (tail partials use the scratch buffer too), again smaller second
    cap = 8
    tails = []
    for a in range(A):
        tk = torch.from_numpy(rng.standard_normal((L, H, cap, d)).astype(np.float16)).cuda()
        tv = torch.from_numpy(rng.standard_normal((L, H, cap, d)).astype(np.float16)).cuda()
        tails.append((tk, tv, 1 + a))
    t_all = pk.Tails(pool, tails)
    out3 = _both(pool, Qd, 0, L, splits=2, tails=t_all)
    t_two = pk.Tails(pool, tails[:2])
    out4 = _both(pool, Q2, 1, 2, splits=0, tails=t_two)
    assert torch.allclose(out4, out3[1:2, :2], atol=1e-3, rtol=0)
    pool.close()


def test_static_entry_point_rejects_what_does_not_fit():
    cfg = W.CONFIGS[5]                                  # 1,024 rows per KV head, 7,194 tokens
    pool = pk.Pool(cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens).bind()
    pool.storage.zero_()
    K = torch.zeros((cfg.layers, cfg.kv_heads, cfg.tokens, cfg.head_dim), dtype=torch.float16, device="cuda:0")
    pool.encode(K, K)
    Q = torch.zeros((cfg.layers, cfg.agents, cfg.q_per_agent, cfg.q_heads, cfg.head_dim), dtype=torch.float16, device="cuda:0")
    out = torch.empty(Q.shape, dtype=torch.float32, device="cuda:0")
    p, _ = pool._params(Q, None, 0, cfg.layers, None, None, pk.KERNEL_AUTO, 0)
    assert pk.lib.pool_attend_workspace(pool._h, C.byref(p)) > pk.STATIC_WORKSPACE_BYTES
    rc = pk.lib.pool_attend_static(pool._h, C.c_void_p(Q.data_ptr()), C.c_void_p(out.data_ptr()), C.byref(p), None)
    assert rc == pk.ENOMEM and b"built-in buffer" in pk.lib.polykv_last_error()
    pool.close()
