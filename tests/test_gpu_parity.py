"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on identical
seeded inputs (shapes and distributions of the workload configurations, reduced in layer count
where the oracle would otherwise take minutes)."""
import math

import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W

pytestmark = pytest.mark.gpu


def _pk():
    from paper_2604_24971_amd import polykv as pk
    return pk


def _pu():
    import parity_util
    return parity_util


class Case:
    """One encoded pool on both sides."""

    def __init__(self, cfg, K=None, V=None, scaled_values=False, int8_values=False, sign_seed=0, key_per_tensor=False,
                 value_bits=3):
        pu = _pu()
        self.cfg = cfg
        if K is None:
            K, V = W.kv_pool(cfg)
        self.K, self.V = K, V
        self.ref = O.pool_encode(K, V, scaled_values=scaled_values, int8_values=int8_values, sign_seed=sign_seed,
                                 key_per_tensor=key_per_tensor, value_bits=value_bits)
        self.pool = pu.gpu_pool(K, V, scaled_values=scaled_values, int8_values=int8_values, sign_seed=sign_seed,
                                key_per_tensor=key_per_tensor, value_bits=value_bits)
        self.dirty, self.k_mis, self.v_mis = pu.compare_codes(self.pool, self.ref)
        self._dec = None

    def decoded(self):
        if self._dec is None:
            self._dec = O.pool_decode(self.ref)
        return self._dec

    def attend_check(self, Q, tails_np=None, tails_len=None, **kw):
        pu = _pu()
        Kh, Vh = self.decoded()
        lb = kw.get("layer_begin", 0)
        le = kw.get("layer_end") or self.cfg.layers
        ref_tails = None
        gpu_tails = None
        if tails_np is not None:
            ref_tails, gpu_tails = [], []
            for (Kt, Vt), n in zip(tails_np, tails_len):
                ref_tails.append((Kt[lb:le, :, :n], Vt[lb:le, :, :n]))
                gpu_tails.append((pu.dev(Kt), pu.dev(Vt), n))
        ref = O.pool_attend(Kh[lb:le], Vh[lb:le], Q, scale=kw.get("scale"), tails=ref_tails)
        out = self.pool.attend(pu.dev(Q), tails=gpu_tails, **kw)
        torch.cuda.synchronize()
        atol = pu.ATTEND_ATOL
        if "v_scales" in self.ref:      # value-codec variants are tested on long vectors: per-row bar
            atol = pu.attend_row_atol(Kh[lb:le], Vh[lb:le], Q, scale=kw.get("scale"), tails=ref_tails)
        return pu.compare_attend(out, ref, self.cfg.kv_heads, self.dirty, lb, atol=atol)


@pytest.fixture(scope="module")
def tiny():
    return Case(W.CONFIGS[1])


@pytest.fixture(scope="module")
def smol():
    return Case(W.CONFIGS[2].scaled(layers=2))


@pytest.fixture(scope="module")
def llama():
    return Case(W.CONFIGS[3].scaled(layers=2, tokens=1500))


# ------------------------------------------------------------------ encode / decode ---
@pytest.mark.parametrize("name", ["tiny", "smol", "llama"])
def test_encode_codes_bit_exact_and_decode_within_tolerance(name, request):
    case = request.getfixturevalue(name)
    pu = _pu()
    n = case.K.size
    assert case.k_mis <= 1e-5 * n and case.v_mis <= 1e-4 * n     # threshold cases are rare
    pu.compare_decode(case.pool, case.ref, case.dirty)
    b = O.stored_bytes(case.cfg.layers, case.cfg.kv_heads, 32 * math.ceil(case.cfg.tokens / 32), case.cfg.head_dim)
    assert case.pool.nbytes == b["packed"]


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("T", [1, 31, 32, 33, 95, 257])
def test_encode_decode_ragged_token_counts(d, T):
    pu = _pu()
    rng = np.random.default_rng(100 * d + T)
    K = (rng.standard_normal((2, 3, T, d)) * np.exp(rng.standard_normal((2, 3, T, 1)))).astype(np.float16)
    V = (rng.standard_normal((2, 3, T, d)) * 1.3).astype(np.float16)
    case = Case(W.PoolConfig(0, "ragged", 2, 3, 6, d, T, 2, 1), K, V)
    pu.compare_decode(case.pool, case.ref, case.dirty)
    Q = rng.standard_normal((2, 2, 1, 6, d)).astype(np.float16)
    case.attend_check(Q)


def test_encode_degenerate_blocks_zero_constant_extreme():
    pu = _pu()
    d, T = 128, 40
    K = np.zeros((1, 2, T, d), dtype=np.float16)
    V = np.zeros_like(K)
    K[0, 0, 3, 32:64] = 0.375                 # constant block -> all +127
    K[0, 0, 4, 5] = -60000.0                  # near fp16 max
    K[0, 0, 5, 64:96] = 6e-8                  # fp16 subnormal input, subnormal scale
    K[0, 1, 7] = np.linspace(-1, 1, d)
    V[0, 0, 2] = 0.25                         # constant vector -> spike at coordinate 0
    V[0, 0, 3, 17] = 8.0                      # spike -> +-8/sqrt(d) everywhere
    V[0, 1, 9] = 300.0                        # saturates the outer centroid
    case = Case(W.PoolConfig(0, "degenerate", 1, 2, 2, d, T, 1, 1), K, V)
    assert case.k_mis == 0 and case.v_mis == 0
    pu.compare_decode(case.pool, case.ref, case.dirty)
    kc, ks, _ = case.pool.export()
    assert int(kc[0, 0, 3, 32:64].min()) == 127 and float(ks[0, 0, 0, 0]) == 0.0
    assert not kc[0, 0, 0].any()


def test_decode_of_a_layer_range_equals_the_slice_of_the_full_decode(llama):
    pk = _pk()
    Kf, Vf = llama.pool.decode(torch.float32)
    for lb, le in ((0, 1), (1, 2), (0, 2)):
        Kl, Vl = llama.pool.decode(torch.float32, layer_begin=lb, layer_end=le)
        assert torch.equal(Kl, Kf[lb:le]) and torch.equal(Vl, Vf[lb:le])
    Kh, _ = llama.pool.decode(torch.float16, layer_begin=1, layer_end=2)
    assert torch.equal(Kh, Kf[1:2].to(torch.float16))
    with pytest.raises(pk.PolyKVError) as e:
        llama.pool.decode(torch.float32, layer_begin=1, layer_end=3)
    assert e.value.status == pk.ESHAPE


def test_reencode_overwrites_and_storage_is_exactly_pool_bytes():
    pu = _pu()
    pk = _pk()
    cfg = W.CONFIGS[1]
    K, V = W.kv_pool(cfg)
    pool = pk.Pool(cfg.layers, cfg.kv_heads, cfg.head_dim, cfg.tokens)
    guard = 4096
    buf = torch.full((pool.nbytes + 2 * guard,), 0x5C, dtype=torch.uint8, device="cuda:0")
    pool.bind(buf[guard:guard + pool.nbytes])
    pool.encode(pu.dev(V), pu.dev(K))          # swapped on purpose, then overwritten
    pool.encode(pu.dev(K), pu.dev(V))
    ref = O.pool_encode(K, V)
    pu.compare_codes(pool, ref)
    assert bool((buf[:guard] == 0x5C).all()) and bool((buf[guard + pool.nbytes:] == 0x5C).all())


# ------------------------------------------------------------------------- attention ---
def test_attend_tiny_whole_config(tiny):
    pk = _pk()
    Q = W.queries(tiny.cfg)
    for kernel in (pk.KERNEL_AUTO, pk.KERNEL_VECTOR):
        tiny.attend_check(Q, kernel=kernel)


def test_attend_smollm2_shape(smol):
    smol.attend_check(W.queries(smol.cfg))


def test_attend_llama_shape_gqa(llama):
    pk = _pk()
    Q = W.queries(llama.cfg)
    llama.attend_check(Q, kernel=pk.KERNEL_VECTOR)
    llama.attend_check(Q)


@pytest.mark.parametrize("splits", [1, 4, 8, 28, 64])
def test_attend_any_split_count_gives_the_same_answer(llama, splits):
    pk = _pk()
    Q = W.queries(llama.cfg)[:1, :3]
    cfg1 = dict(layer_begin=0, layer_end=1, splits=splits)
    llama.attend_check(Q, kernel=pk.KERNEL_VECTOR, **cfg1)
    llama.attend_check(Q, **cfg1)


def test_attend_layer_ranges_scale_and_multi_query(llama):
    rng = np.random.default_rng(77)
    cfg = llama.cfg
    Q = rng.standard_normal((1, 2, 3, cfg.q_heads, cfg.head_dim)).astype(np.float16)
    llama.attend_check(Q, layer_begin=1, layer_end=2)
    llama.attend_check(Q, layer_begin=1, layer_end=2, scale=0.05)


def test_attend_result_does_not_depend_on_other_agents(llama):
    # agent-count invariance (paper, Findings 1 and 5): batching agents must not change any of them
    pu = _pu()
    Q = W.queries(llama.cfg)
    full = llama.pool.attend(pu.dev(Q))
    for sel in ([4], [0, 7, 14]):
        part = llama.pool.attend(pu.dev(Q[:, sel]))
        # a row moves its softmax reference on its own scores only, so this holds bit for bit
        assert torch.equal(part, full[:, sel])


def test_attend_with_private_tails(llama):
    cfg = llama.cfg
    lens = [0, 1, 5, 63, 64, 17, 0, 2, 33, 64, 9, 40, 1, 64, 3][: cfg.agents]
    tails = W.tails(cfg.scaled(cid=4), [64] * cfg.agents)
    Q = W.queries(cfg, step=1)
    llama.attend_check(Q, tails_np=tails, tails_len=lens)
    # a tail of length zero everywhere is the same as no tail
    pu = _pu()
    a = llama.pool.attend(pu.dev(Q))
    b = llama.pool.attend(pu.dev(Q), tails=[(pu.dev(t[0]), pu.dev(t[1]), 0) for t in tails])
    torch.testing.assert_close(a, b, rtol=0, atol=1e-5)     # fused epilogue vs merge kernel


def test_attend_causal_tails_for_multi_token_steps(llama):
    # three new tokens per agent: query i sees the tail up to its own position
    pu = _pu()
    cfg = llama.cfg
    rng = np.random.default_rng(21)
    A, nq = 4, 3
    Q = rng.standard_normal((cfg.layers, A, nq, cfg.q_heads, cfg.head_dim)).astype(np.float16)
    lens = [7, 1, 0, 64]                 # 1 < nq - 1: that agent's first query sees no tail token at all
    tails = W.tails(cfg.scaled(cid=4, agents=A), [64] * A)
    Kh, Vh = llama.decoded()
    ref = O.pool_attend(Kh, Vh, Q, tails=[(t[0][:, :, :n], t[1][:, :, :n]) for t, n in zip(tails, lens)],
                        tail_causal=True)
    gpu_tails = [(pu.dev(t[0]), pu.dev(t[1]), n) for t, n in zip(tails, lens)]
    out = llama.pool.attend(pu.dev(Q), tails=gpu_tails, tail_causal=True)
    torch.cuda.synchronize()
    pu.compare_attend(out, ref, cfg.kv_heads, llama.dirty, 0)
    # the flag matters: without it the earlier queries see more
    plain = llama.pool.attend(pu.dev(Q), tails=gpu_tails)
    assert float((plain - out)[:, 0, 0].abs().max()) > 1e-3
    torch.testing.assert_close(plain[:, :, -1], out[:, :, -1], rtol=0, atol=1e-6)


def test_attend_tails_tiny_d64(tiny):
    cfg = tiny.cfg
    tails = W.tails(cfg, [70, 70, 70])
    tiny.attend_check(W.queries(cfg, step=2), tails_np=tails, tails_len=[70, 0, 13])


@pytest.fixture(scope="module")
def long_pool():
    # the 7,194-token Llama-shaped pool of configurations 4 and 5 (ragged last tile), one layer
    return Case(W.CONFIGS[4].scaled(layers=1))


def test_attend_config4_shape_private_tails_growing_over_decode_steps(long_pool):
    cfg = long_pool.cfg
    tails = W.tails(cfg, [cfg.max_tail] * cfg.agents)
    for step in (1, 23, 64):                 # every agent has produced `step` private tokens
        long_pool.attend_check(W.queries(cfg, step=step), tails_np=tails, tails_len=[step] * cfg.agents)
    long_pool.attend_check(W.queries(cfg))   # step 0: the pool alone
    # one workgroup per KV head over all 225 tiles, as when all 32 layers go in one call
    long_pool.attend_check(W.queries(cfg), splits=1)
    long_pool.attend_check(W.queries(cfg, step=7), tails_np=tails, tails_len=[7] * cfg.agents, splits=1)


def test_attend_config5_shape_1024_rows_per_kv_head(long_pool):
    # 64 agents x 4 queries x 4 query heads per KV head: 16 blocks of 64 rows per unit
    cfg5 = W.CONFIGS[5].scaled(layers=1)
    Q = W.queries(cfg5)
    assert Q.shape[1] * Q.shape[2] * cfg5.group == 1024
    long_pool.attend_check(Q)
    long_pool.attend_check(Q, splits=1)


def test_attend_special_cases_zero_keys_and_dominant_key():
    pu = _pu()
    rng = np.random.default_rng(5)
    d, T = 64, 200
    V = rng.standard_normal((1, 1, T, d)).astype(np.float16)
    K = np.zeros((1, 1, T, d), dtype=np.float16)
    case = Case(W.PoolConfig(0, "zero-k", 1, 1, 2, d, T, 2, 1), K, V)
    Q = rng.standard_normal((1, 2, 1, 2, d)).astype(np.float16)
    out = case.pool.attend(pu.dev(Q)).cpu().numpy()
    _, Vh = case.decoded()
    np.testing.assert_allclose(out[0, 1, 0, 0], Vh[0, 0].mean(0), atol=2e-3)      # uniform weights
    q = Q[0, 0, 0, 0].astype(np.float32)
    K[0, 0, 123] = (40.0 * q / np.linalg.norm(q)).astype(np.float16)
    case = Case(W.PoolConfig(0, "one-hot", 1, 1, 2, d, T, 2, 1), K, V)
    out = case.pool.attend(pu.dev(Q), scale=1.0).cpu().numpy()
    _, Vh = case.decoded()
    np.testing.assert_allclose(out[0, 0, 0, 0], Vh[0, 0, 123], atol=2e-3)         # one dominant key


def test_attend_equals_dense_attention_over_pool_decode_output(llama):
    # property that holds at any size: the fused read path == softmax attention over pool_decode()
    pu = _pu()
    cfg = llama.cfg
    Q = pu.dev(W.queries(cfg, step=3))
    out = llama.pool.attend(Q)
    Kd, Vd = llama.pool.decode(torch.float32)
    G = cfg.group
    q = Q.double().permute(0, 3, 1, 2, 4)                       # [L, qh, A, nq, d]
    k = Kd.double().repeat_interleave(G, dim=1)                 # [L, qh, T, d]
    v = Vd.double().repeat_interleave(G, dim=1)
    s = torch.einsum("lhand,lhtd->lhant", q, k) / math.sqrt(cfg.head_dim)
    ref = torch.einsum("lhant,lhtd->lhand", torch.softmax(s, dim=-1), v).permute(0, 2, 3, 1, 4)
    assert float((out.double() - ref).abs().max()) < 2e-3


def test_attend_error_paths_on_device(tiny):
    pk = _pk()
    pu = _pu()
    Q = pu.dev(W.queries(tiny.cfg))
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pk.PolyKVError) as e:
        tiny.pool.attend(Q, workspace=small)
    assert e.value.status == pk.ENOMEM
    with pytest.raises(pk.PolyKVError) as e:
        tiny.pool.attend(Q[:, :, :, :3].contiguous())            # 3 q heads over 4 kv heads
    assert e.value.status == pk.ESHAPE
    fresh = pk.Pool(1, 4, 64, 600).bind()
    with pytest.raises(pk.PolyKVError) as e:
        fresh.attend(Q)
    assert e.value.status == pk.ESTATE


def test_time_next_kernel_hook_stamps_the_kernel_and_disarms(tiny):
    pk = _pk()
    pu = _pu()
    Q = pu.dev(W.queries(tiny.cfg))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in ev:
        e.record()                       # creates the handles
    torch.cuda.synchronize()
    ref = tiny.pool.attend(Q)
    ev[2].record()
    pk.time_next_kernel(ev[0], ev[1])
    out = tiny.pool.attend(Q)
    again = tiny.pool.attend(Q)          # hook is disarmed: plain launch
    ev[3].record()
    torch.cuda.synchronize()
    kernel_ms, around_ms = ev[0].elapsed_time(ev[1]), ev[2].elapsed_time(ev[3])
    assert 0.0 < kernel_ms < around_ms
    torch.testing.assert_close(out, ref, rtol=0, atol=0)
    torch.testing.assert_close(again, ref, rtol=0, atol=0)


def test_per_layer_calls_captured_in_a_hip_graph_replay_identically(llama):
    # the realistic decode loop: one pool_attend per layer; the library neither allocates nor synchronizes,
    # so the calls can be captured once and replayed
    pu = _pu()
    cfg = llama.cfg
    Q = pu.dev(W.queries(cfg, step=5))
    Ql = [Q[l:l + 1].contiguous() for l in range(cfg.layers)]
    outs = [torch.empty(q.shape, dtype=torch.float32, device=q.device) for q in Ql]
    ws = torch.empty(max(llama.pool.attend_workspace_bytes(Ql[0], layer_begin=0, layer_end=1), 256),
                     dtype=torch.uint8, device=Q.device)

    def decode_step():
        for l in range(cfg.layers):
            llama.pool.attend(Ql[l], outs[l], layer_begin=l, layer_end=l + 1, workspace=ws)

    decode_step()                                   # eager: also configures the kernels before any capture
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    ref = llama.pool.attend(Q)                      # all layers in one call
    torch.testing.assert_close(torch.cat(eager), ref, rtol=0, atol=2e-5)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            decode_step()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        scratch = llama.pool.attend(Q)              # eager work on the same workspace-free path in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), "replay %d differs from the eager result" % rep
        assert torch.equal(scratch, ref)


# --------------------------------------------------------------------- incremental fill ---
@pytest.mark.parametrize("d,chunks", [(128, [37, 1, 90, 32, 5, 64, 27]), (64, [1, 1, 30, 33, 95]),
                                      (128, [32, 64]), (64, [200])])
def test_append_in_chunks_equals_one_encode_of_the_concatenation(d, chunks):
    pk = _pk()
    pu = _pu()
    rng = np.random.default_rng(7 * d + len(chunks))
    Lr, H, cap = 2, 3, sum(chunks) + 40
    T = sum(chunks)
    K = (rng.standard_normal((Lr, H, T, d)) * np.exp(0.7 * rng.standard_normal((Lr, H, T, 1)))).astype(np.float16)
    V = (rng.standard_normal((Lr, H, T, d)) * 1.2).astype(np.float16)
    pool = pk.Pool(Lr, H, d, cap).bind()
    pool.storage.fill_(0xA5)             # stale bytes must never leak into results
    assert pool.length == 0
    Q = rng.standard_normal((Lr, 3, 1, 2 * H, d)).astype(np.float16)
    pos = 0
    for n in chunks:
        pool.append(pu.dev(np.ascontiguousarray(K[:, :, pos:pos + n])), pu.dev(np.ascontiguousarray(V[:, :, pos:pos + n])))
        pos += n
        assert pool.length == pos
        # everything encoded so far equals the oracle's encoding of the prefix, and reads work on it
        ref = O.pool_encode(K[:, :, :pos], V[:, :, :pos])
        dirty, k_mis, v_mis = pu.compare_codes(pool, ref)
        pu.compare_decode(pool, ref, dirty)
        Kh, Vh = O.pool_decode(ref)
        out = pool.attend(pu.dev(Q))
        torch.cuda.synchronize()
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0)
    with pytest.raises(pk.PolyKVError) as e:
        pool.append(pu.dev(np.zeros((Lr, H, 41, d), np.float16)), pu.dev(np.zeros((Lr, H, 41, d), np.float16)))
    assert e.value.status == pk.ESHAPE
    # a full re-encode starts over at the pool's capacity
    Kc = np.concatenate([K, np.zeros((Lr, H, cap - T, d), np.float16)], axis=2)
    Vc = np.concatenate([V, np.zeros((Lr, H, cap - T, d), np.float16)], axis=2)
    pool.encode(pu.dev(Kc), pu.dev(Vc))
    assert pool.length == cap
    pu.compare_codes(pool, O.pool_encode(Kc, Vc))


# ------------------------------------------------------------------------ extreme shapes ---
def test_one_long_head_and_very_many_short_units():
    pu = _pu()
    pk = _pk()
    rng = np.random.default_rng(31)
    # one KV head with 50,001 tokens (1,563 tiles, a ragged last one): many splits, long rows of partials
    T, d = 50001, 64
    K = (rng.standard_normal((1, 1, T, d)) * 0.5).astype(np.float16)
    V = rng.standard_normal((1, 1, T, d)).astype(np.float16)
    case = Case(W.PoolConfig(0, "long", 1, 1, 4, d, T, 3, 1), K, V)
    pu.compare_decode(case.pool, case.ref, case.dirty)
    Q = rng.standard_normal((1, 3, 1, 4, d)).astype(np.float16)
    case.attend_check(Q)
    case.attend_check(Q, splits=1)
    case.attend_check(Q, splits=300)
    # 4,000 (layer, KV head) units of 33 tokens: the unit index fills the grid's second dimension
    L, H, T2 = 500, 8, 33
    K2 = rng.standard_normal((L, H, T2, d)).astype(np.float16)
    V2 = rng.standard_normal((L, H, T2, d)).astype(np.float16)
    case2 = Case(W.PoolConfig(0, "wide", L, H, 8, d, T2, 1, 1), K2, V2)
    pu.compare_decode(case2.pool, case2.ref, case2.dirty)
    Q2 = rng.standard_normal((L, 1, 1, 8, d)).astype(np.float16)
    case2.attend_check(Q2)
    case2.attend_check(Q2[490:], layer_begin=490, layer_end=500, kernel=pk.KERNEL_VECTOR)


@pytest.mark.parametrize("d", [64, 128, 256])
def test_attend_scores_that_keep_climbing_raise_the_softmax_reference_again_and_again(d):
    # Along the pool the scores of some rows grow by more than 2^15 from tile to tile (17 to 18 binary orders:
    # within a tile the probabilities against the old reference overflow fp16), so the matrix kernel has to move
    # its softmax reference (and rescale what it has accumulated) in every step, for those rows only; others rise
    # gently (a move every other tile), stay flat or fall.
    rng = np.random.default_rng(31 + d)
    T, A, qh = 330, 3, 4
    qdir = rng.standard_normal(d)
    qdir /= np.linalg.norm(qdir)
    ramp = np.linspace(0.0, 14.0, T)[:, None]                         # key length along qdir
    K = (ramp * qdir[None, :] + 0.02 * rng.standard_normal((T, d))).astype(np.float16)[None, None]
    V = rng.standard_normal((1, 1, T, d)).astype(np.float16)
    case = Case(W.PoolConfig(0, "climb", 1, 1, qh, d, T, A, 1), K, V)
    # rows: steeply rising (126 nats over the pool: 12 per tile), gently rising, flat, falling
    lengths = np.array([9.0, 4.0, 0.0, -6.0, 9.0, 1.0, -9.0, 0.5, 2.0, 9.0, -1.0, 6.0])
    Q = (lengths[:, None] * qdir[None, :]).astype(np.float16).reshape(1, A, 1, qh, d)
    case.attend_check(Q, scale=1.0, splits=1)
    case.attend_check(Q, scale=1.0)
    case.attend_check(Q, scale=1.0, kernel=_pk().KERNEL_VECTOR)
