"""CPU-only checks of the C-ABI library: it loads, exports every function the header declares,
and its host-side logic (validation, sizes, state machine, codebook) behaves as documented.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from conftest import ROOT
from oracle import polykv_oracle as O

pk = pytest.importorskip("paper_2604_24971_amd.polykv")
lib = pk.lib


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "polykv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:pool|polykv)_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared_functions()
    assert {"pool_create", "pool_bytes", "pool_bind", "pool_encode", "pool_decode", "pool_export",
            "pool_attend_workspace", "pool_attend", "pool_destroy", "polykv_codebook",
            "polykv_last_error", "pool_append", "pool_length", "pool_decode_layers", "polykv_time_next_kernel",
            "pool_create_codec", "pool_export_value_scales", "pool_encode_dtype", "pool_append_dtype", "pool_set_sign_seed", "pool_create_codecs", "polykv_codebook_bits"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_codebook_literals_equal_oracle_codebook_in_fp32():
    c8, t7 = (C.c_float * 8)(), (C.c_float * 7)()
    lib.polykv_codebook(c8, t7)
    for bits in (2, 3, 4):
        c, t = pk.codebook(bits)
        oc, ot = O.codebook(bits)
        np.testing.assert_array_equal(np.array(c, np.float32), oc.astype(np.float32))
        np.testing.assert_array_equal(np.array(t, np.float32), ot.astype(np.float32))
        if bits == 3:
            assert list(c8) == c and list(t7) == t
    assert lib.polykv_codebook_bits(5, None, None) == pk.EINVAL


def _create(L, H, d, T):
    h = C.c_void_p()
    rc = lib.pool_create(L, H, d, T, C.byref(h))
    return rc, h


def test_create_validation_and_byte_counts():
    for bad in [(1, 1, 96, 10), (1, 1, 512, 10), (1, 1, 32, 10), (0, 1, 64, 10), (1, 0, 64, 10), (1, 1, 64, 0),
                (1, 1, 64, -5), (70000, 1, 64, 10), (1, 1, 128, 24_000_000), (1, 1, 64, 2**31 - 1)]:
        rc, h = _create(*bad)
        assert rc == pk.ESHAPE and not h.value
        assert lib.polykv_last_error()
    assert lib.pool_create(1, 1, 64, 1, None) == pk.EINVAL
    rc, h = _create(1, 1, 128, 23_000_000)         # the largest KV heads stay under 4 GiB of records
    assert rc == pk.OK and lib.pool_bytes(h) == 23_000_000 // 32 * 32 * 184
    lib.pool_destroy(h)
    assert lib.pool_bytes(None) == 0
    # tile-multiple token counts: exactly the oracle's stored byte count (184 / 92 B per token-head)
    for (L, H, d, T) in [(32, 8, 128, 4096), (1, 4, 64, 640), (24, 32, 64, 1856), (2, 4, 256, 320)]:
        rc, h = _create(L, H, d, T)
        assert rc == pk.OK
        assert lib.pool_bytes(h) == O.stored_bytes(L, H, T, d)["packed"]
        lib.pool_destroy(h)
    # ragged token counts are padded to whole tiles of 32
    rc, h = _create(32, 8, 128, 7194)
    assert lib.pool_bytes(h) == O.stored_bytes(32, 8, 7200, 128)["packed"]
    lib.pool_destroy(h)
    lib.pool_destroy(None)


def test_value_codec_choice_byte_counts_and_errors():
    h = C.c_void_p()
    assert lib.pool_create_codec(1, 1, 64, 10, 7, C.byref(h)) == pk.EINVAL and not h.value
    for codec, bits, scaled in [(pk.VALUES_TQ2, 2, False), (pk.VALUES_TQ2_SCALED, 2, True), (pk.VALUES_TQ4, 4, False),
                                (pk.VALUES_TQ4_SCALED, 4, True)]:
        for (L, H, d, T) in [(32, 8, 128, 4096), (1, 4, 64, 640), (2, 2, 256, 64)]:
            assert lib.pool_create_codec(L, H, d, T, codec, C.byref(h)) == pk.OK
            assert lib.pool_bytes(h) == O.stored_bytes(L, H, T, d, scaled_values=scaled, value_bits=bits)["packed"]
            lib.pool_destroy(h)
    for (L, H, d, T) in [(32, 8, 128, 4096), (1, 4, 64, 640)]:
        assert lib.pool_create_codec(L, H, d, T, pk.VALUES_TQ3_SCALED, C.byref(h)) == pk.OK
        assert lib.pool_bytes(h) == O.stored_bytes(L, H, T, d, scaled_values=True)["packed"]
        lib.pool_destroy(h)
        assert lib.pool_create_codec(L, H, d, T, pk.VALUES_INT8, C.byref(h)) == pk.OK
        assert lib.pool_bytes(h) == O.stored_bytes(L, H, T, d, int8_values=True)["packed"]
        lib.pool_destroy(h)
        assert lib.pool_create_codec(L, H, d, T, pk.VALUES_TQ3, C.byref(h)) == pk.OK
        assert lib.pool_bytes(h) == O.stored_bytes(L, H, T, d)["packed"]
        lib.pool_destroy(h)
    fake = C.c_void_p(0x10000)       # never dereferenced
    assert lib.pool_create_codec(1, 1, 64, 10, pk.VALUES_TQ3_SCALED, C.byref(h)) == pk.OK
    assert lib.pool_export_value_scales(h, fake, None) == pk.ESTATE   # nothing bound / encoded
    assert lib.pool_set_sign_seed(h, 12345) == pk.OK and lib.pool_set_sign_seed(h, 0) == pk.OK
    assert lib.pool_set_sign_seed(None, 1) == pk.EINVAL
    lib.pool_destroy(h)
    # one key scale per layer tensor: no per-block scales, the layers' maxima behind the records; no append
    assert lib.pool_create_codecs(1, 1, 64, 10, 5, pk.VALUES_TQ3, C.byref(h)) == pk.EINVAL
    assert lib.pool_create_codecs(32, 8, 128, 4096, pk.KEYS_Q8_TENSOR, pk.VALUES_TQ3, C.byref(h)) == pk.OK
    assert lib.pool_bytes(h) == 32 * 8 * 4096 * 176 + 256
    assert lib.pool_bind(h, fake, lib.pool_bytes(h)) == pk.OK
    assert lib.pool_append(h, fake, fake, 5, None) == pk.ESTATE
    lib.pool_destroy(h)
    assert lib.pool_create_codec(1, 1, 64, 10, pk.VALUES_INT8, C.byref(h)) == pk.OK
    assert lib.pool_set_sign_seed(h, 12345) == pk.ESTATE              # int8 values are not rotated
    assert lib.pool_set_sign_seed(h, 0) == pk.OK
    lib.pool_destroy(h)


def test_state_machine_and_argument_errors_without_gpu():
    rc, h = _create(2, 2, 64, 100)
    assert rc == pk.OK
    fake = C.c_void_p(0x10000)       # never dereferenced: every call below fails validation first
    assert lib.pool_encode(h, fake, fake, None) == pk.ESTATE          # nothing bound
    assert lib.pool_decode(h, fake, fake, pk.F32, None) == pk.ESTATE
    assert lib.pool_export(h, fake, fake, fake, None) == pk.ESTATE
    assert lib.pool_bind(h, None, 1 << 30) == pk.EINVAL
    assert lib.pool_bind(h, C.c_void_p(0x10010), 1 << 30) == pk.EINVAL  # misaligned
    assert lib.pool_bind(h, fake, 10) == pk.ENOMEM
    assert b"needed" in lib.polykv_last_error()
    assert lib.pool_bind(None, fake, 10) == pk.EINVAL
    assert lib.pool_bind(h, fake, lib.pool_bytes(h)) == pk.OK
    assert lib.pool_encode(h, None, fake, None) == pk.EINVAL
    assert lib.pool_encode_dtype(h, fake, fake, pk.F32, None) == pk.EINVAL    # fp16 or bfloat16 only
    assert lib.pool_append_dtype(h, fake, fake, 5, 9, None) == pk.EINVAL
    assert lib.pool_encode(h, C.c_void_p(0x10002), fake, None) == pk.EINVAL   # misaligned input
    # bound but not encoded: reads refuse
    assert lib.pool_decode(h, fake, fake, pk.F32, None) == pk.ESTATE
    p = pk.AttendParams()
    p.agents, p.q_per_agent, p.q_heads, p.layer_begin, p.layer_end = 3, 1, 2, 0, 2
    assert lib.pool_attend(h, fake, fake, C.byref(p), None) == pk.ESTATE
    assert b"not been encoded" in lib.polykv_last_error()
    # incremental fill: an empty pool after bind, capacity checked before anything is launched
    assert lib.pool_length(h) == 0 and lib.pool_length(None) == 0
    assert lib.pool_append(h, fake, fake, 101, None) == pk.ESHAPE
    assert b"do not fit" in lib.polykv_last_error()
    assert lib.pool_append(h, fake, fake, 0, None) == pk.ESHAPE
    assert lib.pool_append(h, None, fake, 5, None) == pk.EINVAL
    assert lib.pool_append(None, fake, fake, 5, None) == pk.EINVAL
    assert lib.pool_length(h) == 0
    lib.pool_destroy(h)
    rc, h = _create(1, 1, 64, 10)
    assert lib.pool_append(h, fake, fake, 5, None) == pk.ESTATE           # nothing bound
    lib.pool_destroy(h)


def test_attend_plan_validation_and_workspace_size():
    rc, h = _create(4, 2, 128, 4000)
    p = pk.AttendParams()
    p.agents, p.q_per_agent, p.q_heads, p.layer_begin, p.layer_end = 3, 1, 8, 0, 4
    need = lib.pool_attend_workspace(h, C.byref(p))
    assert need > 0 and need % 256 == 0
    # at least one partial (m, l, acc[d]) per row per split
    rows = 3 * 1 * 4
    assert need >= 4 * 2 * rows * (128 + 2) * 4
    p.splits = 8
    need8 = lib.pool_attend_workspace(h, C.byref(p))
    p.splits = 16
    assert lib.pool_attend_workspace(h, C.byref(p)) > need8
    p.splits = 0
    for field, val in [("q_heads", 7), ("agents", 0), ("q_per_agent", 0), ("layer_end", 5),
                       ("layer_begin", 4), ("kernel", 9), ("splits", -1), ("io_dtype", pk.F32), ("io_dtype", 7)]:
        q = pk.AttendParams.from_buffer_copy(p)
        setattr(q, field, val)
        assert lib.pool_attend_workspace(h, C.byref(q)) == 0, field
        assert lib.polykv_last_error()
    assert lib.pool_attend_workspace(h, None) == 0
    assert lib.pool_attend_workspace(None, C.byref(p)) == 0
    # tails: lengths are checked against the capacity, agent count against the maximum
    tl = (C.c_int * 3)(1, 5, 0)
    tk = (C.c_void_p * 3)(0x1000, 0x2000, 0)
    q = pk.AttendParams.from_buffer_copy(p)
    q.tail_K = C.cast(tk, C.POINTER(C.c_void_p))
    q.tail_V = C.cast(tk, C.POINTER(C.c_void_p))
    q.tail_len = C.cast(tl, C.POINTER(C.c_int))
    q.tail_capacity = 4
    assert lib.pool_attend_workspace(h, C.byref(q)) == 0
    q.tail_capacity = 8
    assert lib.pool_attend_workspace(h, C.byref(q)) > need
    # launch limits: 4-row blocks of the vector and tail kernels sit on grid.z (65,535 at most)
    big = pk.AttendParams.from_buffer_copy(p)
    big.agents, big.q_per_agent = 1, 65536                       # 262,144 rows per KV head
    assert lib.pool_attend_workspace(h, C.byref(big)) > 0        # fine for the matrix kernel
    big.kernel = pk.KERNEL_VECTOR
    assert lib.pool_attend_workspace(h, C.byref(big)) == 0
    assert b"262,140" in lib.polykv_last_error()
    q.q_per_agent = 65536
    assert lib.pool_attend_workspace(h, C.byref(q)) == 0
    big.kernel, big.q_per_agent = pk.KERNEL_AUTO, (1 << 18) + 1   # more than 2^20 rows
    assert lib.pool_attend_workspace(h, C.byref(big)) == 0
    for bad in (-1.0, float("nan"), float("inf")):
        q = pk.AttendParams.from_buffer_copy(p)
        q.scale = bad
        assert lib.pool_attend_workspace(h, C.byref(q)) == 0, bad
    lib.pool_destroy(h)


def test_python_binding_rejects_wrong_tensors_before_any_launch():
    import torch
    pool = pk.Pool(1, 2, 64, 50)
    assert pool.nbytes == 2 * 2 * 2944
    with pytest.raises(TypeError):
        pool.bind(torch.empty(pool.nbytes, dtype=torch.uint8))        # CPU tensor
    with pytest.raises(ValueError):
        pool.encode(torch.empty(1, 2, 49, 64), torch.empty(1, 2, 49, 64))
    pool.close()
    with pytest.raises(pk.PolyKVError):
        pk.Pool(1, 2, 80, 50)


def test_header_is_valid_c99(tmp_path):
    # the boundary is a C ABI: the header must compile as plain C, on its own
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_polykv.c"
    src.write_text('#include "polykv.h"\n'
                   "int use(void) { polykv_attend_params p = {0}; polykv_pool* h = 0;\n"
                   "  return pool_create_codecs(1, 1, 64, 1, POLYKV_KEYS_Q8_BLOCK32, POLYKV_VALUES_TQ3, &h) + p.agents\n"
                   "         + (int)sizeof(polykv_status) + POLYKV_BF16 + POLYKV_KERNEL_AUTO; }\n")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_bench_command_line_refuses_more_than_one_gpu_and_malformed_phases():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    bench = os.path.join(root, "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
    r = subprocess.run([sys.executable, bench, "--phases", "ee"], capture_output=True, text=True)
    assert r.returncode != 0 and "--phases" in r.stderr
