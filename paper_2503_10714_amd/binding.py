"""ctypes binding of libzsm.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/zsm.h).  Tensors are
torch tensors on the GPU; the binding passes their data pointers and the current HIP
stream.  There is no fallback: if the library has not been built the import of this
module's `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzsm.so")

ZSM_F32, ZSM_F16, ZSM_BF16 = 0, 1, 2
DTYPE_CODE = {torch.float32: ZSM_F32, torch.float16: ZSM_F16, torch.bfloat16: ZSM_BF16,
              "f32": ZSM_F32, "f16": ZSM_F16, "bf16": ZSM_BF16}
CODE_TORCH = {ZSM_F32: torch.float32, ZSM_F16: torch.float16, ZSM_BF16: torch.bfloat16}

EXPORTS = [
    "zsm_cache_bytes", "zsm_cache_alloc", "zsm_cache_free", "zsm_prefill_workspace_bytes",
    "zsm_prefill_compress", "zsm_decode_step", "zsm_decode_step_static", "zsm_cache_set_decode_parts", "zsm_decode_parts",
    "zsm_cache_export", "zsm_cache_import", "zsm_cache_flags", "zsm_set_debug_checks",
    "zsm_stream_read", "zsm_stream_copy", "zsm_strerror",
]


class zsm_config_t(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_seqs", C.c_int32), ("n_kv_heads", C.c_int32),
                ("q_per_kv", C.c_int32), ("head_dim", C.c_int32), ("slot_capacity", C.c_int32),
                ("n_residual", C.c_int32), ("kv_dtype", C.c_int32),
                ("lambda_", C.c_float), ("alpha", C.c_float), ("scale", C.c_float)]


class ZsmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {zsm_strerror(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.zsm_cache_bytes.restype = sz
        L.zsm_cache_bytes.argtypes = [C.POINTER(zsm_config_t)]
        L.zsm_cache_alloc.restype = C.c_int
        L.zsm_cache_alloc.argtypes = [C.POINTER(zsm_config_t), C.POINTER(i32), C.POINTER(i32), vp, sz, vp, C.POINTER(vp)]
        L.zsm_cache_free.restype = C.c_int
        L.zsm_cache_free.argtypes = [vp]
        L.zsm_prefill_workspace_bytes.restype = sz
        L.zsm_prefill_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.zsm_prefill_compress.restype = C.c_int
        L.zsm_prefill_compress.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, i32, vp, sz, vp]
        L.zsm_decode_step.restype = C.c_int
        L.zsm_decode_step.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.zsm_decode_step_static.restype = C.c_int
        L.zsm_decode_step_static.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.zsm_cache_set_decode_parts.restype = C.c_int
        L.zsm_cache_set_decode_parts.argtypes = [vp, i32]
        L.zsm_decode_parts.restype = C.c_int
        L.zsm_decode_parts.argtypes = [vp, i32, i32]
        L.zsm_cache_export.restype = C.c_int
        L.zsm_cache_export.argtypes = [vp, i32] + [vp] * 8 + [vp]
        L.zsm_cache_import.restype = C.c_int
        L.zsm_cache_import.argtypes = [vp, i32] + [vp] * 8 + [vp]
        L.zsm_cache_flags.restype = C.c_int
        L.zsm_cache_flags.argtypes = [vp, i32, vp, i32, vp]
        L.zsm_set_debug_checks.restype = C.c_int
        L.zsm_set_debug_checks.argtypes = [i32]
        L.zsm_stream_read.restype = C.c_int
        L.zsm_stream_read.argtypes = [vp, sz, vp, vp]
        L.zsm_stream_copy.restype = C.c_int
        L.zsm_stream_copy.argtypes = [vp, vp, sz, vp]
        L.zsm_strerror.restype = C.c_char_p
        L.zsm_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise ZsmError(rc, where)


def zsm_strerror(status: int) -> str:
    return lib().zsm_strerror(int(status)).decode()


def make_config(n_layers, n_seqs, n_kv_heads, q_per_kv, head_dim, slot_capacity, n_residual, kv_dtype,
                lam=0.98, alpha=1.0, scale=0.0) -> zsm_config_t:
    return zsm_config_t(n_layers, n_seqs, n_kv_heads, q_per_kv, head_dim, slot_capacity, n_residual,
                        DTYPE_CODE[kv_dtype], lam, alpha, scale)


def zsm_cache_bytes(cfg: zsm_config_t) -> int:
    return int(lib().zsm_cache_bytes(C.byref(cfg)))


def zsm_cache_alloc(cfg: zsm_config_t, B_p: Sequence[int], B_c: Sequence[int], dev_buf: torch.Tensor, stream=None):
    n = cfg.n_seqs
    if len(B_p) != n or len(B_c) != n:
        raise ValueError("B_p and B_c need one entry per sequence")
    bp = (C.c_int32 * n)(*[int(x) for x in B_p])
    bc = (C.c_int32 * n)(*[int(x) for x in B_c])
    out = C.c_void_p()
    rc = lib().zsm_cache_alloc(C.byref(cfg), bp, bc, _ptr(dev_buf), dev_buf.numel() * dev_buf.element_size(),
                               _stream(stream), C.byref(out))
    _check(rc, "zsm_cache_alloc")
    return out


def zsm_cache_free(handle) -> None:
    _check(lib().zsm_cache_free(handle), "zsm_cache_free")


def zsm_prefill_workspace_bytes(handle, n_layers: int, T_max: int, W: int) -> int:
    return int(lib().zsm_prefill_workspace_bytes(handle, n_layers, T_max, W))


def zsm_prefill_compress(handle, layer_begin, layer_end, Q, W, K, V, seq_lens, T_max, workspace, stream=None) -> None:
    rc = lib().zsm_prefill_compress(handle, layer_begin, layer_end, _ptr(Q), W, _ptr(K), _ptr(V), _ptr(seq_lens), T_max,
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "zsm_prefill_compress")


def zsm_decode_step(handle, layer_begin, layer_end, q, k_new, v_new, out, write_slot=None, evicted_pos=None,
                    merged_slot=None, stream=None) -> None:
    rc = lib().zsm_decode_step(handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                               _ptr(write_slot), _ptr(evicted_pos), _ptr(merged_slot), _stream(stream))
    _check(rc, "zsm_decode_step")


def zsm_decode_step_static(handle, layer_begin, layer_end, q, k_new, v_new, out, write_slot=None, evicted_pos=None,
                           merged_slot=None, stream=None) -> None:
    rc = lib().zsm_decode_step_static(handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                      _ptr(write_slot), _ptr(evicted_pos), _ptr(merged_slot), _stream(stream))
    _check(rc, "zsm_decode_step_static")


def zsm_cache_set_decode_parts(handle, parts: int) -> None:
    _check(lib().zsm_cache_set_decode_parts(handle, int(parts)), "zsm_cache_set_decode_parts")


def zsm_decode_parts(handle, layer_begin: int, layer_end: int) -> int:
    rc = int(lib().zsm_decode_parts(handle, int(layer_begin), int(layer_end)))
    if rc < 0:
        raise ZsmError(rc, "zsm_decode_parts")
    return rc


def zsm_cache_export(handle, layer, K=None, V=None, Kr=None, Vr=None, s=None, pos=None, w=None, n_seen=None, stream=None):
    rc = lib().zsm_cache_export(handle, layer, _ptr(K), _ptr(V), _ptr(Kr), _ptr(Vr), _ptr(s), _ptr(pos), _ptr(w),
                                _ptr(n_seen), _stream(stream))
    _check(rc, "zsm_cache_export")


def zsm_cache_import(handle, layer, K=None, V=None, Kr=None, Vr=None, s=None, pos=None, w=None, n_seen=None, stream=None):
    rc = lib().zsm_cache_import(handle, layer, _ptr(K), _ptr(V), _ptr(Kr), _ptr(Vr), _ptr(s), _ptr(pos), _ptr(w),
                                _ptr(n_seen), _stream(stream))
    _check(rc, "zsm_cache_import")


def zsm_cache_flags(handle, layer, flags=None, clear=False, stream=None) -> None:
    _check(lib().zsm_cache_flags(handle, int(layer), _ptr(flags), 1 if clear else 0, _stream(stream)), "zsm_cache_flags")


def zsm_set_debug_checks(on) -> int:
    return int(lib().zsm_set_debug_checks(1 if on else 0))


def zsm_stream_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    _check(lib().zsm_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)), "zsm_stream_read")


def zsm_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    _check(lib().zsm_stream_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)), "zsm_stream_copy")


class Cache:
    """Convenience owner of one cache: holds the torch buffer and the C descriptor, allocates
    output tensors.  Every step still runs in the library's kernels."""

    def __init__(self, n_layers, n_seqs, n_kv_heads, q_per_kv, head_dim, B_p, B_c, n_residual, kv_dtype,
                 lam=0.98, alpha=1.0, scale=0.0, slot_capacity=None, device="cuda:0"):
        self.device = torch.device(device)
        B_p = [int(B_p)] * n_seqs if isinstance(B_p, int) else [int(x) for x in B_p]
        B_c = [int(B_c)] * n_seqs if isinstance(B_c, int) else [int(x) for x in B_c]
        cap = max(p + c for p, c in zip(B_p, B_c)) + n_residual if slot_capacity is None else slot_capacity
        self.cfg = make_config(n_layers, n_seqs, n_kv_heads, q_per_kv, head_dim, cap, n_residual, kv_dtype,
                               lam, alpha, scale)
        self.kv_dtype = CODE_TORCH[self.cfg.kv_dtype]
        self.B_p, self.B_c = B_p, B_c
        nbytes = zsm_cache_bytes(self.cfg)
        if nbytes == 0:
            raise ZsmError(-2, "zsm_cache_bytes")
        with torch.cuda.device(self.device):
            self.buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.handle = zsm_cache_alloc(self.cfg, B_p, B_c, self.buf)
        self._ws = None

    def close(self):
        if getattr(self, "handle", None) is not None:
            zsm_cache_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # shapes ---------------------------------------------------------------------------
    @property
    def L(self): return self.cfg.n_layers
    @property
    def S(self): return self.cfg.n_seqs
    @property
    def H(self): return self.cfg.n_kv_heads
    @property
    def G(self): return self.cfg.q_per_kv
    @property
    def d(self): return self.cfg.head_dim
    @property
    def cap(self): return self.cfg.slot_capacity
    @property
    def B_r(self): return self.cfg.n_residual

    def prefill_compress(self, layer: int, Q, K, V, seq_lens, layer_end: Optional[int] = None) -> None:
        """One layer (Q [S,H,G,W,d], K/V [S,H,T,d]) or, with layer_end, the layers [layer, layer_end) in one call
        (Q [Ln,S,H,G,W,d], K/V [Ln,S,H,T,d])."""
        S, H, G, d = self.S, self.H, self.G, self.d
        W, T_max = Q.shape[-2], K.shape[-2]
        lead = () if layer_end is None else (layer_end - layer,)
        layer_end = layer + 1 if layer_end is None else layer_end
        assert tuple(Q.shape) == lead + (S, H, G, W, d) and tuple(K.shape) == lead + (S, H, T_max, d) and K.shape == V.shape
        assert Q.dtype == self.kv_dtype and K.dtype == self.kv_dtype and V.dtype == self.kv_dtype
        if not torch.is_tensor(seq_lens):
            seq_lens = torch.tensor(list(seq_lens), dtype=torch.int32)
        seq_lens = seq_lens.to(device=self.device, dtype=torch.int32).contiguous()
        self.reserve_workspace(layer_end - layer, T_max, W)
        with torch.cuda.device(self.device):
            zsm_prefill_compress(self.handle, layer, layer_end, Q, W, K, V, seq_lens, T_max, self._ws)

    def reserve_workspace(self, n_layers: int, T_max: int, W: int) -> None:
        """Hold a workspace large enough for prefill calls of `n_layers` layers (allocated here, ahead of the call,
        by whoever does not want the allocation inside a timed region)."""
        need = zsm_prefill_workspace_bytes(self.handle, n_layers, T_max, W)
        if need == 0:
            raise ZsmError(-2, "zsm_prefill_workspace_bytes")
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)

    def release_workspace(self):
        self._ws = None

    def decode_step(self, q, k_new, v_new, layer_begin=0, layer_end=None, out=None, info=None):
        """info: None -> allocate the three int32 outputs; False -> skip them; or a tuple of tensors."""
        layer_end = self.L if layer_end is None else layer_end
        Ln = layer_end - layer_begin
        S, H, G, d = self.S, self.H, self.G, self.d
        assert tuple(q.shape) == (Ln, S, H, G, d) and tuple(k_new.shape) == (Ln, S, H, d) and k_new.shape == v_new.shape
        assert q.dtype == self.kv_dtype and k_new.dtype == self.kv_dtype and v_new.dtype == self.kv_dtype
        if out is None:
            out = torch.empty(Ln, S, H, G, d, dtype=torch.float32, device=self.device)
        if info is None:
            info = tuple(torch.empty(Ln, S, H, dtype=torch.int32, device=self.device) for _ in range(3))
        ws, ep, ms = info if info else (None, None, None)
        with torch.cuda.device(self.device):
            zsm_decode_step(self.handle, layer_begin, layer_end, q, k_new, v_new, out, ws, ep, ms)
        return out, info

    def set_decode_parts(self, parts: int) -> None:
        zsm_cache_set_decode_parts(self.handle, parts)

    def decode_parts(self, layer_begin=0, layer_end=None) -> int:
        return zsm_decode_parts(self.handle, layer_begin, self.L if layer_end is None else layer_end)

    def flags(self, layer: int, clear: bool = False) -> torch.Tensor:
        """The layer's sticky condition bits, int32 [S, H] (device tensor)."""
        out = torch.empty(self.S, self.H, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            zsm_cache_flags(self.handle, layer, out, clear)
        return out

    def export_layer(self, layer: int) -> dict:
        S, H, d, cap, Br = self.S, self.H, self.d, self.cap, self.B_r
        dev = self.device
        st = dict(
            K=torch.empty(S, H, cap - Br, d, dtype=self.kv_dtype, device=dev),
            V=torch.empty(S, H, cap - Br, d, dtype=self.kv_dtype, device=dev),
            Kr=torch.empty(S, H, Br, d, dtype=torch.float32, device=dev),
            Vr=torch.empty(S, H, Br, d, dtype=torch.float32, device=dev),
            s=torch.empty(S, H, cap, dtype=torch.float32, device=dev),
            pos=torch.empty(S, H, cap, dtype=torch.int32, device=dev),
            w=torch.empty(S, H, cap, dtype=torch.int32, device=dev),
            n_seen=torch.empty(S, H, dtype=torch.int64, device=dev),
        )
        with torch.cuda.device(dev):
            zsm_cache_export(self.handle, layer, **st)
        return st

    def import_layer(self, layer: int, **st) -> None:
        st = {k: (v.to(self.device).contiguous() if v is not None else None) for k, v in st.items()}
        with torch.cuda.device(self.device):
            zsm_cache_import(self.handle, layer, **st)
        torch.cuda.synchronize(self.device)   # the staged tensors above may be temporaries
