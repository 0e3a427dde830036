import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden_path(name):
    return os.path.join(ROOT, "tests", "golden", name)


def read_golden_rows(name):
    rows = []
    with open(golden_path(name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def oracle():
    from oracle import polykv_oracle
    return polykv_oracle


# ---- guard bands: every buffer the GPU tests let the binding allocate for a kernel to write into (decode
# outputs, attention output and workspace, exports) gets a margin of a known pattern on both sides, checked
# after the call -- a kernel that writes past either end of its buffer fails the test that ran it.
GUARD_BYTES = 4096
GUARD_BYTE = 0x5C


class _Guarded:
    def __init__(self):
        self.live = []

    def alloc(self, shape, dtype, device):
        import torch
        n = 1
        for x in shape:
            n *= int(x)
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        pad = (-nbytes) % 256
        raw = torch.full((GUARD_BYTES + nbytes + pad + GUARD_BYTES,), GUARD_BYTE, dtype=torch.uint8, device=device)
        view = raw[GUARD_BYTES:GUARD_BYTES + nbytes].view(dtype).view(tuple(int(x) for x in shape))
        self.live.append((raw, nbytes))
        return view

    def check(self, what):
        import torch
        torch.cuda.synchronize()
        for raw, nbytes in self.live:
            head, tail = raw[:GUARD_BYTES], raw[GUARD_BYTES + nbytes:]
            assert bool((head == GUARD_BYTE).all()) and bool((tail == GUARD_BYTE).all()), \
                "%s wrote outside its %d-byte buffer" % (what, nbytes)
        self.live = []


@pytest.fixture(autouse=True)
def _guard_bands(request, monkeypatch):
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    import torch
    from paper_2604_24971_amd import polykv as pk
    g = _Guarded()
    orig_decode, orig_attend, orig_export, orig_scales = pk.Pool.decode, pk.Pool.attend, pk.Pool.export, pk.Pool.export_value_scales

    def decode(self, dtype=torch.float32, K_out=None, V_out=None, stream=None, layer_begin=0, layer_end=None):
        le = self.layers if layer_end is None else layer_end
        shape = (max(le - layer_begin, 0), self.kv_heads, self.length, self.head_dim)
        if K_out is None:
            K_out = g.alloc(shape, dtype, self.device)
        if V_out is None:
            V_out = g.alloc(shape, dtype, self.device)
        r = orig_decode(self, dtype, K_out, V_out, stream, layer_begin, layer_end)
        g.check("pool_decode")
        return r

    def attend(self, Q, out=None, *, workspace=None, stream=None, **kw):
        capturing = torch.cuda.is_current_stream_capturing()
        if not capturing and stream is None:
            if out is None:
                out = g.alloc(Q.shape, torch.float32, self.device)
            if workspace is None:
                need = self.attend_workspace_bytes(Q, **kw)
                if need:
                    workspace = g.alloc((need,), torch.uint8, self.device)
        r = orig_attend(self, Q, out, workspace=workspace, stream=stream, **kw)
        if not capturing and stream is None:
            g.check("pool_attend")
        return r

    monkeypatch.setattr(pk.Pool, "decode", decode)
    monkeypatch.setattr(pk.Pool, "attend", attend)
    yield
