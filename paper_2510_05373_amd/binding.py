"""ctypes binding of libkvlinc.so.  Same names and argument order as include/kvlinc.h."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(HERE, "libkvlinc.so")

KVLINC_OK, KVLINC_EINVAL, KVLINC_EWORKSPACE, KVLINC_EHIP, KVLINC_ESCRATCH = 0, -1, -2, -3, -4
KVLINC_STATIC_SCRATCH_BYTES = 16 << 20
KVLINC_FLAG_ALG1_LITERAL = 1
KVLINC_FLAG_SLIDING_VALUES = 2
KVLINC_ST_CAPACITY, KVLINC_ST_NONFINITE, KVLINC_ST_STATIC, KVLINC_ST_STATE_RANGE = 1, 2, 4, 8


class KVLincError(RuntimeError):
    pass


class CacheStruct(ctypes.Structure):
    """Mirror of struct kvlinc_cache."""
    _fields_ = [
        ("B", ctypes.c_int32), ("H_q", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("G", ctypes.c_int32), ("R", ctypes.c_int32), ("D", ctypes.c_int32), ("bits", ctypes.c_int32),
        ("max_groups", ctypes.c_int64),
        ("groups", ctypes.c_void_p),
        ("k_res", ctypes.c_void_p), ("v_res", ctypes.c_void_p),
        ("n_quant", ctypes.c_void_p), ("n_res", ctypes.c_void_p),
        ("S", ctypes.c_void_p), ("S16", ctypes.c_void_p), ("P", ctypes.c_void_p),
        ("Wq", ctypes.c_void_p), ("Wk", ctypes.c_void_p),
        ("status", ctypes.c_void_p), ("split_done", ctypes.c_void_p),
        ("flags", ctypes.c_int32),
    ]


def _load():
    if not os.path.exists(lib_path):
        raise ImportError(
            "libkvlinc.so is not built (%s missing): run `python -c 'import __graft_entry__ as g; g.build()'` or "
            "`python paper_2510_05373_amd/build.py`; there is no fallback path" % lib_path)
    # PyTorch carries its own copy of the HIP runtime under the same soname as the system one, and the first copy
    # loaded serves the whole process.  The tensors and streams passed to this library come from torch, so torch's
    # runtime has to be that copy: import torch before the library is opened.
    import torch  # noqa: F401
    L = ctypes.CDLL(lib_path)
    P = ctypes.POINTER(CacheStruct)
    L.kvlinc_version.restype = ctypes.c_int
    L.kvlinc_version.argtypes = []
    L.kvlinc_strerror.restype = ctypes.c_char_p
    L.kvlinc_strerror.argtypes = [ctypes.c_int]
    L.kvlinc_cache_validate.restype = ctypes.c_int
    L.kvlinc_cache_validate.argtypes = [P]
    L.kvlinc_append_quantize.restype = ctypes.c_int
    L.kvlinc_append_quantize.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_void_p]
    L.kvlinc_decode_workspace_bytes.restype = ctypes.c_size_t
    L.kvlinc_decode_workspace_bytes.argtypes = [P, ctypes.c_int32]
    L.kvlinc_decode_attention.restype = ctypes.c_int
    L.kvlinc_decode_attention.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                          ctypes.c_int32, ctypes.c_void_p]
    L.kvlinc_decode_attention_timed.restype = ctypes.c_int
    L.kvlinc_decode_attention_timed.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    L.kvlinc_decode_attention_noalloc.restype = ctypes.c_int
    L.kvlinc_decode_attention_noalloc.argtypes = [P, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
    return L


lib = _load()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _struct(cache):
    return cache.struct if isinstance(cache, KVLincCache) else cache


def kvlinc_version():
    return lib.kvlinc_version()


def kvlinc_strerror(code):
    return lib.kvlinc_strerror(code).decode()


def kvlinc_cache_validate(cache):
    return lib.kvlinc_cache_validate(ctypes.byref(_struct(cache)))


def kvlinc_append_quantize(cache, k_new, v_new, n_new=None, T=None, keep_residual=0, stream=None):
    """k_new, v_new: [B, H_kv, T, 128] fp16 device tensors (contiguous); n_new: [B] int32 device tensor or None."""
    if T is None:
        T = k_new.shape[2]
    return lib.kvlinc_append_quantize(ctypes.byref(_struct(cache)), _ptr(k_new), _ptr(v_new), _ptr(n_new), int(T),
                                      int(keep_residual), _stream(stream))


def kvlinc_decode_workspace_bytes(cache, max_context=0):
    return lib.kvlinc_decode_workspace_bytes(ctypes.byref(_struct(cache)), int(max_context))


def kvlinc_decode_attention(cache, q, out, workspace, workspace_bytes=None, max_context=0, stream=None):
    """q, out: [B, H_q, 128] fp16 device tensors; workspace: device tensor of at least the advertised bytes."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib.kvlinc_decode_attention(ctypes.byref(_struct(cache)), _ptr(q), _ptr(out), _ptr(workspace),
                                       int(workspace_bytes), int(max_context), _stream(stream))


def kvlinc_decode_attention_timed(cache, q, out, workspace, start_event, stop_event, workspace_bytes=None,
                                  max_context=0, stream=None):
    """As kvlinc_decode_attention; start_event / stop_event are raw hipEvent_t handles (integers)."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib.kvlinc_decode_attention_timed(ctypes.byref(_struct(cache)), _ptr(q), _ptr(out), _ptr(workspace),
                                             int(workspace_bytes), int(max_context), _stream(stream),
                                             ctypes.c_void_p(int(start_event)), ctypes.c_void_p(int(stop_event)))


def kvlinc_decode_attention_noalloc(cache, q, out, max_context=0, stream=None):
    """As kvlinc_decode_attention, with the library's static scratch buffer in place of a workspace."""
    return lib.kvlinc_decode_attention_noalloc(ctypes.byref(_struct(cache)), _ptr(q), _ptr(out), int(max_context),
                                               _stream(stream))


class KVLincCache:
    """Device buffers of one layer's cache plus the descriptor that points at them (allocation only)."""

    def __init__(self, B, H_q, H_kv, max_context, R=128, Wq=None, Wk=None, device="cuda", state_storage="fp32",
                 flags=0, bits=2):
        """state_storage: "fp32" keeps the fp32 master copy of S next to its binary16 tiles, "fp16" stores the state in
        the binary16 tiles only; flags: KVLINC_FLAG_* bits; bits: width of the codes, 2 or 4 (group records of 2304 or
        4352 words)."""
        import torch
        assert bits in (2, 4)
        self.B, self.H_q, self.H_kv, self.R, self.bits = B, H_q, H_kv, R, bits
        self.max_groups = max(1, -(-int(max_context) // 128))
        dev = torch.device(device)
        mg = self.max_groups
        z = lambda *s, dt: torch.zeros(*s, dtype=dt, device=dev)
        self.groups = z(B, H_kv, mg, 2304 if bits == 2 else 4352, dt=torch.int32)
        self.k_res = z(B, H_kv, R, 128, dt=torch.float16)
        self.v_res = z(B, H_kv, R // 4, 128, 4, dt=torch.float16)
        self.n_quant = z(B, dt=torch.int32)
        self.n_res = z(B, dt=torch.int32)
        self.status = z(1, dt=torch.int32)
        self.split_done = z(B, H_kv, dt=torch.int32)
        self.Wq, self.Wk = Wq, Wk
        if Wq is not None:
            assert Wk is not None and tuple(Wq.shape) == (H_q, 2, 128, 128) and tuple(Wk.shape) == (H_kv, 2, 128, 128)
            assert Wq.dtype == torch.float16 and Wk.dtype == torch.float16 and Wq.is_contiguous() and Wk.is_contiguous()
            assert state_storage in ("fp32", "fp16")
            self.S = z(B, H_kv, 256, 128, dt=torch.float32) if state_storage == "fp32" else None
            self.S16 = z(B, H_kv, 128, 64, 4, dt=torch.float16)
            self.P = z(B, H_kv, 256, dt=torch.float32)
        else:
            self.S = self.S16 = self.P = None
        self.struct = CacheStruct(
            B=B, H_q=H_q, H_kv=H_kv, d=128, G=128, R=R, D=256, bits=bits, max_groups=mg,
            groups=self.groups.data_ptr(),
            k_res=self.k_res.data_ptr(), v_res=self.v_res.data_ptr(),
            n_quant=self.n_quant.data_ptr(), n_res=self.n_res.data_ptr(),
            S=None if self.S is None else self.S.data_ptr(), S16=None if self.S16 is None else self.S16.data_ptr(),
            P=None if self.P is None else self.P.data_ptr(),
            Wq=None if Wq is None else Wq.data_ptr(), Wk=None if Wk is None else Wk.data_ptr(),
            status=self.status.data_ptr(), split_done=self.split_done.data_ptr(), flags=int(flags))
        self._ws = None

    def bytes(self):
        ts = [self.groups, self.k_res, self.v_res]
        if self.S16 is not None:
            ts += [self.S16, self.P] + ([self.S] if self.S is not None else [])
        return sum(t.numel() * t.element_size() for t in ts)

    def append(self, k_new, v_new, n_new=None, keep_residual=0, stream=None):
        rc = kvlinc_append_quantize(self, k_new, v_new, n_new, k_new.shape[2], keep_residual, stream)
        if rc != KVLINC_OK:
            raise KVLincError("kvlinc_append_quantize: " + kvlinc_strerror(rc))

    def workspace(self, max_context=0):
        import torch
        need = kvlinc_decode_workspace_bytes(self, max_context)
        if self._ws is None or self._ws.numel() * 4 < need:
            self._ws = torch.empty((need + 3) // 4, dtype=torch.float32, device=self.groups.device)
        return self._ws

    def decode(self, q, out=None, max_context=0, stream=None):
        import torch
        if out is None:
            out = torch.empty_like(q)
        ws = self.workspace(max_context)
        rc = kvlinc_decode_attention(self, q, out, ws, ws.numel() * 4, max_context, stream)
        if rc != KVLINC_OK:
            raise KVLincError("kvlinc_decode_attention: " + kvlinc_strerror(rc))
        return out
