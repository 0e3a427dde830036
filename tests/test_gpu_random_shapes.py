"""Seeded random sweeps over shapes, codecs and call options against the oracle: whatever combination the
hand-written cases leave out (head_dim x rows per KV head x token count x codec x sign diagonal x key codec x
splits x kernel x tails; chunked appends x bfloat16 inputs)."""
import numpy as np
import pytest
import torch

from oracle import polykv_oracle as O
from paper_2604_24971_amd import workloads as W
from test_gpu_parity import Case, _pk, _pu

pytestmark = pytest.mark.gpu

CODECS = ["tq3", "scaled", "int8", "tq2", "tq4", "tq2s", "tq4s"]


def _codec_kw(codec):
    return dict(scaled_values=codec in ("scaled", "tq2s", "tq4s"), int8_values=codec == "int8",
                value_bits={"tq2": 2, "tq2s": 2, "tq4": 4, "tq4s": 4}.get(codec, 3))


def _kv(rng, L, H, T, d, wide):
    K = rng.standard_normal((L, H, T, d)) * np.exp(0.5 * rng.standard_normal((L, H, 1, d)))
    V = rng.standard_normal((L, H, T, d)) * np.exp((1.0 if wide else 0.3) * rng.standard_normal((L, H, T, 1)))
    return K, V


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_pools_and_attention_calls(seed):
    pu, pk = _pu(), _pk()
    rng = np.random.default_rng(seed)
    for _ in range(40):
        d = int(rng.choice([64, 128, 256]))
        L, H, G = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 4, 5]))
        T = int(rng.choice([1, 7, 31, 32, 33, 64, 95, 129, 300, 777][: (8 if d == 256 else 10)]))
        A, nq = int(rng.integers(1, 18)), int(rng.choice([1, 1, 1, 2, 3]))
        codec = str(rng.choice(CODECS))
        kw = _codec_kw(codec)
        sign_seed = int(rng.integers(0, 3)) if codec != "int8" else 0
        kpt = bool(rng.integers(0, 4) == 0)
        K, V = _kv(rng, L, H, T, d, kw["scaled_values"] or kw["int8_values"])
        what = "d=%d L=%d H=%d G=%d T=%d A=%d nq=%d %s sign=%d tensor-keys=%d" % (d, L, H, G, T, A, nq, codec, sign_seed, kpt)
        print(what, flush=True)
        case = Case(W.PoolConfig(0, "random", L, H, H * G, d, T, A, nq), K.astype(np.float16), V.astype(np.float16),
                    sign_seed=sign_seed, key_per_tensor=kpt, **kw)
        pu.compare_decode(case.pool, case.ref, case.dirty)
        Q = rng.standard_normal((L, A, nq, H * G, d)).astype(np.float16)
        case.attend_check(Q)
        case.attend_check(Q, splits=int(rng.choice([1, 2, 3, 7])))
        if T <= 129 and A * nq * G <= 40:
            case.attend_check(Q, kernel=pk.KERNEL_VECTOR)
        if A <= 15 and rng.integers(0, 2):
            cap = int(rng.choice([1, 5, 40]))
            tails = [(rng.standard_normal((L, H, cap, d)).astype(np.float16), rng.standard_normal((L, H, cap, d)).astype(np.float16))
                     for _ in range(A)]
            case.attend_check(Q, tails_np=tails, tails_len=[int(rng.integers(0, cap + 1)) for _ in range(A)])


@pytest.mark.parametrize("seed", [11, 12])
def test_random_chunked_appends_fp16_and_bfloat16(seed):
    pu, pk = _pu(), _pk()
    rng = np.random.default_rng(seed)
    for _ in range(60):
        d = int(rng.choice([64, 128, 256]))
        L, H, G = int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.choice([1, 2, 4]))
        chunks = [int(rng.choice([1, 2, 5, 31, 32, 33, 64, 70])) for _ in range(int(rng.integers(1, 6)))]
        T = sum(chunks)
        cap = T + int(rng.integers(0, 40))
        codec = str(rng.choice(CODECS))
        kw = _codec_kw(codec)
        sign_seed = int(rng.integers(0, 3)) if codec != "int8" else 0
        bf16 = bool(rng.integers(0, 3) == 0)
        K, V = _kv(rng, L, H, T, d, kw["scaled_values"] or kw["int8_values"])
        K, V = (W.bf16_round(K.astype(np.float32)), W.bf16_round(V.astype(np.float32))) if bf16 else (K.astype(np.float16), V.astype(np.float16))
        print("d=%d L=%d H=%d G=%d chunks=%s capacity=%d %s sign=%d bf16=%d" % (d, L, H, G, chunks, cap, codec, sign_seed, bf16), flush=True)
        pool = pk.Pool(L, H, d, cap, value_codec=pu.value_codec_id(**kw), sign_seed=sign_seed).bind()
        pool.storage.fill_(0xA5)
        pos = 0
        for c in chunks:
            pool.append(pu.dev(np.ascontiguousarray(K[:, :, pos:pos + c]), bf16), pu.dev(np.ascontiguousarray(V[:, :, pos:pos + c]), bf16))
            pos += c
        ref = O.pool_encode(K, V, sign_seed=sign_seed, **kw)
        if kw["scaled_values"]:
            pu.settle_value_scales(pool.export_value_scales().cpu().numpy(), ref)
        dirty, _, _ = pu.compare_codes(pool, ref)
        pu.compare_decode(pool, ref, dirty)
        Kh, Vh = O.pool_decode(ref)
        Q = rng.standard_normal((L, int(rng.integers(1, 8)), 1, H * G, d)).astype(np.float16)
        out = pool.attend(pu.dev(Q))
        torch.cuda.synchronize()
        wide = kw["scaled_values"] or kw["int8_values"]      # the paper's codec keeps the fixed bar, bfloat16 inputs too
        pu.compare_attend(out, O.pool_attend(Kh, Vh, Q), H, dirty, 0, atol=pu.attend_row_atol(Kh, Vh, Q) if wide else pu.ATTEND_ATOL)
