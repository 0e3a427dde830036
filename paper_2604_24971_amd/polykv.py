"""ctypes binding of libpolykv.so: argument marshalling only -- every step of the hot path runs in
the HIP kernels behind the C ABI declared in include/polykv.h.  torch supplies device memory and
the current stream, nothing else.  Importing this module fails loudly if the library is missing."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpolykv.so")

OK, EINVAL, ESHAPE, ESTATE, ENOMEM, EHIP = 0, -1, -2, -3, -4, -5
F16, F32, BF16 = 0, 1, 2
_DTYPES = {torch.float16: F16, torch.float32: F32, torch.bfloat16: BF16}
KERNEL_AUTO, KERNEL_VECTOR, KERNEL_MATRIX = 0, 1, 2
KEY_PRECISION_EXACT, KEY_PRECISION_FP16 = 0, 1
VALUES_TQ3, VALUES_TQ3_SCALED, VALUES_INT8 = 0, 1, 2
VALUES_TQ2, VALUES_TQ2_SCALED, VALUES_TQ4, VALUES_TQ4_SCALED = 3, 4, 5, 6
VALUE_BITS = {0: 3, 1: 3, 2: 8, 3: 2, 4: 2, 5: 4, 6: 4}
KEYS_Q8_BLOCK32, KEYS_Q8_TENSOR = 0, 1
MAX_TAIL_AGENTS = 64
STATIC_WORKSPACE_BYTES = 32 << 20


class PolyKVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("polykv status %d: %s" % (status, message))
        self.status = status


class AttendParams(C.Structure):
    _fields_ = [
        ("agents", C.c_int), ("q_per_agent", C.c_int), ("q_heads", C.c_int),
        ("layer_begin", C.c_int), ("layer_end", C.c_int), ("scale", C.c_float),
        ("tail_K", C.POINTER(C.c_void_p)), ("tail_V", C.POINTER(C.c_void_p)),
        ("tail_len", C.POINTER(C.c_int)), ("tail_capacity", C.c_int), ("tail_causal", C.c_int),
        ("kernel", C.c_int), ("splits", C.c_int),
        ("workspace_dev", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("io_dtype", C.c_int), ("key_precision", C.c_int),
    ]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libpolykv.so is not built (%s); run `python -m paper_2604_24971_amd.build`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, ip, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.pool_create.argtypes = [ip, ip, ip, ip, C.POINTER(vp)]
    lib.pool_create.restype = ip
    lib.pool_create_codec.argtypes = [ip, ip, ip, ip, ip, C.POINTER(vp)]
    lib.pool_create_codec.restype = ip
    lib.pool_create_codecs.argtypes = [ip, ip, ip, ip, ip, ip, C.POINTER(vp)]
    lib.pool_create_codecs.restype = ip
    lib.pool_set_sign_seed.argtypes = [vp, C.c_uint64]
    lib.pool_set_sign_seed.restype = ip
    lib.pool_destroy.argtypes = [vp]
    lib.pool_destroy.restype = None
    lib.pool_bytes.argtypes = [vp]
    lib.pool_bytes.restype = sz
    lib.pool_bind.argtypes = [vp, vp, sz]
    lib.pool_bind.restype = ip
    lib.pool_encode.argtypes = [vp, vp, vp, vp]
    lib.pool_encode.restype = ip
    lib.pool_append.argtypes = [vp, vp, vp, ip, vp]
    lib.pool_append.restype = ip
    lib.pool_encode_dtype.argtypes = [vp, vp, vp, ip, vp]
    lib.pool_encode_dtype.restype = ip
    lib.pool_append_dtype.argtypes = [vp, vp, vp, ip, ip, vp]
    lib.pool_append_dtype.restype = ip
    lib.pool_length.argtypes = [vp]
    lib.pool_length.restype = ip
    lib.pool_decode_layers.argtypes = [vp, vp, vp, ip, ip, ip, vp]
    lib.pool_decode_layers.restype = ip
    lib.pool_decode.argtypes = [vp, vp, vp, ip, vp]
    lib.pool_decode.restype = ip
    lib.pool_export.argtypes = [vp, vp, vp, vp, vp]
    lib.pool_export.restype = ip
    lib.pool_export_value_scales.argtypes = [vp, vp, vp]
    lib.pool_export_value_scales.restype = ip
    lib.pool_attend_workspace.argtypes = [vp, C.POINTER(AttendParams)]
    lib.pool_attend_workspace.restype = sz
    lib.pool_attend.argtypes = [vp, vp, vp, C.POINTER(AttendParams), vp]
    lib.pool_attend.restype = ip
    lib.pool_attend_static.argtypes = [vp, vp, vp, C.POINTER(AttendParams), vp]
    lib.pool_attend_static.restype = ip
    lib.polykv_codebook.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.polykv_codebook.restype = None
    lib.polykv_codebook_bits.argtypes = [ip, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.polykv_codebook_bits.restype = ip
    lib.polykv_time_next_kernel.argtypes = [vp, vp]
    lib.polykv_time_next_kernel.restype = ip
    lib.polykv_last_error.argtypes = []
    lib.polykv_last_error.restype = C.c_char_p
    return lib


lib = _load()


def _check(rc: int):
    if rc != OK:
        raise PolyKVError(rc, lib.polykv_last_error().decode())


def codebook(bits: int = 3):
    c = (C.c_float * (1 << bits))()
    t = (C.c_float * ((1 << bits) - 1))()
    _check(lib.polykv_codebook_bits(bits, c, t))
    return list(c), list(t)


def time_next_kernel(start: torch.cuda.Event, stop: torch.cuda.Event):
    """polykv_time_next_kernel(start, stop): the next encode / decode / attend call of this thread stamps the two
    events at the begin and end of its main kernel.  The events must have been recorded once before, so
    that torch has created their handles."""
    _check(lib.polykv_time_next_kernel(C.c_void_p(start.cuda_event), C.c_void_p(stop.cuda_event)))


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dev_ptr(t: torch.Tensor, dtype, what: str):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (what, dtype))
    return C.c_void_p(t.data_ptr())


class Tails:
    """The agents' private continuations, marshalled once: per agent a (K, V) pair of fp16 tensors
    [layers, kv_heads, capacity, head_dim] (or None) that the caller keeps appending to, plus the current
    lengths, which set_lengths() updates in place between decode steps."""

    def __init__(self, pool: "Pool", tensors, lengths=None):
        A = len(tensors)
        if A > MAX_TAIL_AGENTS:
            raise ValueError("at most %d agents can carry private tails" % MAX_TAIL_AGENTS)
        self.agents = A
        self.k = (C.c_void_p * A)()
        self.v = (C.c_void_p * A)()
        self.len = (C.c_int * A)()
        self.capacity = 0
        self.dtype = None            # torch.float16 or torch.bfloat16, the same for every tail
        self._keep = []
        for a, ent in enumerate(tensors):
            if ent is None:
                continue
            Kt, Vt = ent[0], ent[1]
            shape = (pool.layers, pool.kv_heads, Kt.shape[2], pool.head_dim)
            if tuple(Kt.shape) != shape or tuple(Vt.shape) != shape:
                raise ValueError("tail tensors must be [layers, kv_heads, capacity, head_dim]")
            if self.capacity and self.capacity != Kt.shape[2]:
                raise ValueError("all tails must share one capacity")
            self.capacity = Kt.shape[2]
            if self.dtype is None:
                self.dtype = Kt.dtype
            if self.dtype not in (torch.float16, torch.bfloat16):
                raise TypeError("tails must be float16 or bfloat16")
            self.k[a] = _dev_ptr(Kt, self.dtype, "tail K").value
            self.v[a] = _dev_ptr(Vt, self.dtype, "tail V").value
            self._keep += [Kt, Vt]
            if len(ent) > 2:
                self.len[a] = int(ent[2])
        if lengths is not None:
            self.set_lengths(lengths)

    def set_lengths(self, lengths):
        if len(lengths) != self.agents:
            raise ValueError("one length per agent")
        for a, n in enumerate(lengths):
            self.len[a] = int(n)
        return self


class Pool:
    """pool_create + pool_bind around a torch-owned storage tensor."""

    def __init__(self, layers: int, kv_heads: int, head_dim: int, tokens: int, device="cuda:0",
                 value_codec: int = VALUES_TQ3, sign_seed: int = 0, key_codec: int = KEYS_Q8_BLOCK32):
        self.layers, self.kv_heads, self.head_dim, self.tokens = layers, kv_heads, head_dim, tokens
        self.value_codec = value_codec
        self.key_codec = key_codec
        self.device = torch.device(device)
        h = C.c_void_p()
        _check(lib.pool_create_codecs(layers, kv_heads, head_dim, tokens, key_codec, value_codec, C.byref(h)))
        self._h = h
        if sign_seed:
            _check(lib.pool_set_sign_seed(self._h, sign_seed))
        self.nbytes = lib.pool_bytes(self._h)
        self.storage = None
        self._workspaces = {}   # stream handle -> cached attend workspace

    def bind(self, storage: torch.Tensor | None = None):
        if storage is None:
            storage = torch.empty(self.nbytes, dtype=torch.uint8, device=self.device)
        _check(lib.pool_bind(self._h, _dev_ptr(storage, torch.uint8, "storage"), storage.numel()))
        self.storage = storage
        return self

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:      # `lib` is already gone when the interpreter shuts down
            lib.pool_destroy(h)

    __del__ = close

    # pool_encode(K, V)
    def encode(self, K: torch.Tensor, V: torch.Tensor, stream=None):
        shape = (self.layers, self.kv_heads, self.tokens, self.head_dim)
        if tuple(K.shape) != shape or tuple(V.shape) != shape:
            raise ValueError("K and V must have shape %s" % (shape,))
        if K.dtype not in (torch.float16, torch.bfloat16):
            raise TypeError("K and V must be float16 or bfloat16")
        _check(lib.pool_encode_dtype(self._h, _dev_ptr(K, K.dtype, "K"), _dev_ptr(V, K.dtype, "V"), _DTYPES[K.dtype],
                                     _stream_ptr(stream)))

    # pool_append(K, V, count)
    def append(self, K: torch.Tensor, V: torch.Tensor, stream=None):
        if K.dim() != 4 or tuple(K.shape) != tuple(V.shape) or \
                tuple(K.shape[:2]) != (self.layers, self.kv_heads) or K.shape[3] != self.head_dim:
            raise ValueError("K and V must be [layers, kv_heads, count, head_dim]")
        if K.dtype not in (torch.float16, torch.bfloat16):
            raise TypeError("K and V must be float16 or bfloat16")
        _check(lib.pool_append_dtype(self._h, _dev_ptr(K, K.dtype, "K"), _dev_ptr(V, K.dtype, "V"),
                                     int(K.shape[2]), _DTYPES[K.dtype], _stream_ptr(stream)))

    @property
    def length(self) -> int:
        return lib.pool_length(self._h)

    # pool_decode(K_out, V_out)
    def decode(self, dtype=torch.float32, K_out=None, V_out=None, stream=None, layer_begin=0, layer_end=None):
        layer_end = self.layers if layer_end is None else layer_end
        shape = (max(layer_end - layer_begin, 0), self.kv_heads, self.length, self.head_dim)
        code = _DTYPES[dtype]
        if K_out is None:
            K_out = torch.empty(shape, dtype=dtype, device=self.device)
        if V_out is None:
            V_out = torch.empty(shape, dtype=dtype, device=self.device)
        if tuple(K_out.shape) != shape or tuple(V_out.shape) != shape:
            raise ValueError("decode outputs must have shape %s" % (shape,))
        _check(lib.pool_decode_layers(self._h, _dev_ptr(K_out, dtype, "K_out"), _dev_ptr(V_out, dtype, "V_out"),
                                      code, layer_begin, layer_end, _stream_ptr(stream)))
        return K_out, V_out

    def export(self, stream=None):
        n = (self.layers, self.kv_heads, self.length)
        kc = torch.empty(n + (self.head_dim,), dtype=torch.int8, device=self.device)
        if self.key_codec == KEYS_Q8_TENSOR:     # one scale per layer tensor
            ks = torch.empty((self.layers,), dtype=torch.float16, device=self.device)
        else:
            ks = torch.empty(n + (self.head_dim // 32,), dtype=torch.float16, device=self.device)
        if self.value_codec == VALUES_INT8:      # the int8 value codes themselves
            vp = torch.empty(n + (self.head_dim,), dtype=torch.int8, device=self.device)
        else:
            vp = torch.empty(n + (VALUE_BITS[self.value_codec] * self.head_dim // 8,), dtype=torch.uint8, device=self.device)
        _check(lib.pool_export(self._h, C.c_void_p(kc.data_ptr()), C.c_void_p(ks.data_ptr()),
                               C.c_void_p(vp.data_ptr()), _stream_ptr(stream)))
        return kc, ks, vp

    def export_value_scales(self, stream=None):
        vs = torch.empty((self.layers, self.kv_heads, self.length), dtype=torch.float16, device=self.device)
        _check(lib.pool_export_value_scales(self._h, C.c_void_p(vs.data_ptr()), _stream_ptr(stream)))
        return vs

    def _params(self, Q, q_heads, layer_begin, layer_end, scale, tails, kernel, splits, tail_causal=False,
                key_precision=KEY_PRECISION_EXACT):
        if Q.dim() != 5:
            raise ValueError("Q must be [layers_selected, agents, q_per_agent, q_heads, head_dim]")
        layer_end = self.layers if layer_end is None else layer_end
        Ls, A, nq, qh, d = Q.shape
        if Ls != layer_end - layer_begin or d != self.head_dim or (q_heads is not None and qh != q_heads):
            raise ValueError("Q shape %s does not match the layer range / head_dim" % (tuple(Q.shape),))
        p = AttendParams()
        p.agents, p.q_per_agent, p.q_heads = A, nq, qh
        p.layer_begin, p.layer_end, p.scale = layer_begin, layer_end, float(scale or 0.0)
        p.kernel, p.splits = kernel, splits
        p.key_precision = key_precision
        if Q.dtype not in (torch.float16, torch.bfloat16):
            raise TypeError("Q must be float16 or bfloat16")
        p.io_dtype = _DTYPES[Q.dtype]
        keep = []
        if tails is not None:
            if not isinstance(tails, Tails):
                tails = Tails(self, tails)
            if tails.agents != A:
                raise ValueError("tails must have one entry per agent")
            if tails.dtype is not None and tails.dtype != Q.dtype:
                raise TypeError("Q and the tails must have the same dtype")
            p.tail_K = C.cast(tails.k, C.POINTER(C.c_void_p))
            p.tail_V = C.cast(tails.v, C.POINTER(C.c_void_p))
            p.tail_len = C.cast(tails.len, C.POINTER(C.c_int))
            p.tail_capacity = tails.capacity
            p.tail_causal = 1 if tail_causal else 0
            keep.append(tails)
        return p, keep

    def attend_workspace_bytes(self, Q, **kw):
        p, _keep = self._params(Q, kw.get("q_heads"), kw.get("layer_begin", 0), kw.get("layer_end"),
                                kw.get("scale"), kw.get("tails"), kw.get("kernel", KERNEL_AUTO),
                                kw.get("splits", 0), kw.get("tail_causal", False))
        return lib.pool_attend_workspace(self._h, C.byref(p))

    # pool_attend(Q[agents], out)
    def attend(self, Q: torch.Tensor, out: torch.Tensor | None = None, *, q_heads=None, layer_begin=0,
               layer_end=None, scale=None, tails=None, kernel=KERNEL_AUTO, splits=0, workspace=None,
               stream=None, tail_causal=False, key_precision=KEY_PRECISION_EXACT):
        p, _keep = self._params(Q, q_heads, layer_begin, layer_end, scale, tails, kernel, splits, tail_causal,
                                key_precision)
        need = lib.pool_attend_workspace(self._h, C.byref(p))
        if need == 0:
            _check(lib.pool_attend(self._h, None, None, C.byref(p), None))  # surfaces the shape error
        if workspace is None:
            # one cached workspace per stream: calls on different streams may overlap and must not share one
            key = _stream_ptr(stream).value
            ws = self._workspaces.get(key)
            if ws is None or ws.numel() < need:
                ws = self._workspaces[key] = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
            workspace = ws
        p.workspace_dev = _dev_ptr(workspace, torch.uint8, "workspace")
        p.workspace_bytes = workspace.numel()
        if out is None:
            out = torch.empty(Q.shape, dtype=torch.float32, device=self.device)
        _check(lib.pool_attend(self._h, _dev_ptr(Q, Q.dtype, "Q"), _dev_ptr(out, torch.float32, "out"),
                               C.byref(p), _stream_ptr(stream)))
        return out

    # pool_attend_static(Q[agents], out): no workspace, nothing allocated by the library
    def attend_static(self, Q: torch.Tensor, out: torch.Tensor, *, q_heads=None, layer_begin=0, layer_end=None,
                      scale=None, tails=None, kernel=KERNEL_AUTO, splits=0, stream=None, tail_causal=False,
                      key_precision=KEY_PRECISION_EXACT):
        p, _keep = self._params(Q, q_heads, layer_begin, layer_end, scale, tails, kernel, splits, tail_causal,
                                key_precision)
        _check(lib.pool_attend_static(self._h, _dev_ptr(Q, Q.dtype, "Q"), _dev_ptr(out, torch.float32, "out"),
                                      C.byref(p), _stream_ptr(stream)))
        return out
