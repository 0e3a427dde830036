"""One KV head of 20 million tokens: its packed records take 3.7 GB, so tile offsets pass 2^31 bytes and come
close to the 4 GiB that pool_create allows per KV head.  The oracle cannot run at this size; instead the three
entry points are checked against each other and against the input, with the attention mass placed on the last
100,000 tokens, i.e. on the records at the largest offsets:
  * decode against the input (quantization error statistics of the method, there and at the pool's start),
  * attend against plain torch attention over the decoded tensors (a different addressing path)."""
import math

import pytest
import torch

pytestmark = pytest.mark.gpu


def test_twenty_million_token_head_addresses_beyond_two_gib():
    from paper_2604_24971_amd import polykv as pk

    if torch.cuda.get_device_properties(0).total_memory < 60 * 2**30:
        pytest.skip("needs about 30 GB of device memory")
    d, T, hot = 128, 20_000_017, 100_000
    g = torch.Generator(device="cuda")
    g.manual_seed(20)
    qdir = torch.randn(d, device="cuda", generator=g)
    qdir /= qdir.norm()
    K = torch.randn(1, 1, T, d, device="cuda", generator=g, dtype=torch.float16)
    K *= 0.05
    K[0, 0, T - hot:] += (16.0 * qdir).to(torch.float16)          # the last tokens carry the attention mass
    V = torch.randn(1, 1, T, d, device="cuda", generator=g, dtype=torch.float16)
    # 2 agents x 2 query heads on the one KV head: 4 rows, all looking along qdir with different lengths
    Q = (qdir[None, :] * torch.tensor([8.0, 7.0, 6.0, 9.0], device="cuda")[:, None]).to(torch.float16)
    Q = Q.reshape(1, 2, 1, 2, d).contiguous()

    pool = pk.Pool(1, 1, d, T).bind()
    assert pool.nbytes > 3 * 2**30
    pool.encode(K, V)
    out = pool.attend(Q)
    Kh, Vh = pool.decode(torch.float16)
    torch.cuda.synchronize()

    # decode against the input where the offsets are largest: keys within half a quantization step of the
    # block scale, values with the codebook's relative error (0.0345 for unit-variance coordinates)
    lo = T - hot
    Kt, Kht = K[0, 0, lo:].float(), Kh[0, 0, lo:].float()
    step = Kt.reshape(hot, d // 32, 32).abs().amax(-1) / 127.0
    assert ((Kht - Kt).reshape(hot, d // 32, 32).abs().amax(-1) <= 0.5 * step * 1.01 + 1e-3).all()
    Vt, Vht = V[0, 0, lo:].float(), Vh[0, 0, lo:].float()
    rel = ((Vht - Vt) ** 2).sum() / (Vt ** 2).sum()
    assert 0.030 < float(rel) < 0.040
    # ... and at the start of the pool
    rel0 = ((Vh[0, 0, :hot].float() - V[0, 0, :hot].float()) ** 2).sum() / (V[0, 0, :hot].float() ** 2).sum()
    assert 0.030 < float(rel0) < 0.040

    # attention over the decoded tensors in plain torch
    q = Q.reshape(4, d).float()
    s = (Kh[0, 0].float() @ q.t()) / math.sqrt(d)                    # [T, 4]
    p = torch.softmax(s, dim=0)
    assert float(p[lo:].sum(0).min()) > 0.95                         # the mass does sit on the last tokens
    ref = (p.t() @ Vh[0, 0].float()).reshape(1, 2, 1, 2, d)
    assert float((out - ref).abs().max()) <= 3e-3
    assert float(out.abs().max()) > 1e-3
