"""Thin ctypes binding over libh1bkv.so (include/h1bkv.h): same names, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch appears only as the owner of device
memory and streams (`.data_ptr()`, `torch.cuda.current_stream().cuda_stream`).  There is no fallback:
if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

H1BKV_F32, H1BKV_F16 = 0, 1
H1BKV_OK = 0
H1BKV_EINVAL, H1BKV_ENULL, H1BKV_ESHAPE, H1BKV_ENOSPACE = -1, -2, -3, -4
H1BKV_ERANGE, H1BKV_EWORKSPACE, H1BKV_EHIP, H1BKV_ENODEVICE = -5, -6, -7, -8
H1BKV_DEVICE_NONE = -1
H1BKV_PAGE_TOKENS = 256
H1BKV_STATIC_SCRATCH_BYTES = 16 << 20
H1BKV_K_APPEND, H1BKV_K_QSKETCH, H1BKV_K_DECODE_SPLIT, H1BKV_K_MERGE, H1BKV_K_PREFILL = 0, 1, 2, 3, 4

# H1BKV_LIBRARY names another build of the same library (a debug or experimental build); default: the in-tree one
LIB_PATH = os.environ.get("H1BKV_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libh1bkv.so")


class h1bkv_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_q_heads", "n_kv_heads", "head_dim", "sketch_bits", "group_size", "in_dtype",
                                         "page_tokens", "max_seqs", "max_pages", "max_pages_per_seq", "device", "value_bits")]
    _fields_ += [("seed", C.c_uint64)]


class H1BKVError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {h1bkv_strerror(code)} ({code})")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load the built library (raises if it is missing: there is no CPU path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2510_05529_amd.build`")
        # PyTorch ships its own libamdhip64; load it first so that this library binds to the same HIP runtime
        # (two runtimes in one process do not see each other's allocations, streams or current device).
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        pcfg = C.POINTER(h1bkv_config)
        sig = {
            "h1bkv_version": (C.c_int, []),
            "h1bkv_strerror": (C.c_char_p, [C.c_int]),
            "h1bkv_pool_bytes": (sz, [pcfg]),
            "h1bkv_create": (C.c_int, [pcfg, vp, sz, vp, C.POINTER(vp)]),
            "h1bkv_destroy": (C.c_int, [vp]),
            "h1bkv_get_projection": (C.c_int, [vp, vp]),
            "h1bkv_seq_len": (C.c_int, [vp, i32, C.POINTER(i32)]),
            "h1bkv_free_pages": (C.c_int, [vp, C.POINTER(i32)]),
            "h1bkv_reset_seq": (C.c_int, [vp, i32]),
            "h1bkv_truncate_seq": (C.c_int, [vp, i32, i32]),
            "h1bkv_append_kv": (C.c_int, [vp, vp, i32, i32, vp, vp, i64, i64, i64, vp]),
            "h1bkv_decode_workspace_bytes": (sz, [vp, i32, i32]),
            "h1bkv_decode_attn": (C.c_int, [vp, vp, i32, vp, C.c_float, vp, vp, sz, vp]),
            "h1bkv_decode_attn_static": (C.c_int, [vp, vp, i32, vp, C.c_float, vp, vp]),
            "h1bkv_decode_step": (C.c_int, [vp, vp, i32, vp, vp, i64, i64, vp, C.c_float, vp, vp, sz, vp]),
            "h1bkv_reserve_seq": (C.c_int, [vp, i32, i32, vp]),
            "h1bkv_reserved_tokens": (C.c_int, [vp, i32, C.POINTER(C.c_int32)]),
            "h1bkv_decode_step_dev": (C.c_int, [vp, vp, i32, vp, vp, i64, i64, vp, C.c_float, vp, vp, i32, i32, vp, sz, vp]),
            "h1bkv_set_seq_len": (C.c_int, [vp, i32, i32]),
            "h1bkv_decode_dtau_workspace_bytes": (sz, [vp, i32, i32]),
            "h1bkv_decode_attn_dtau": (C.c_int, [vp, vp, i32, vp, C.c_float, vp, vp, vp, sz, vp]),
            "h1bkv_prefill_workspace_bytes": (sz, [vp, i32, i32]),
            "h1bkv_prefill_attn": (C.c_int, [vp, vp, i32, i32, vp, i64, i64, i64, C.c_float, vp, vp, sz, vp]),
            "h1bkv_set_decode_chunk": (C.c_int, [vp, i32]),
            "h1bkv_set_projection_path": (C.c_int, [vp, i32]),
            "h1bkv_debug_fail_launch": (C.c_int, [vp, i32]),
            "h1bkv_export_tokens": (C.c_int, [vp, i32, i32, i32, i32, vp, vp, vp, vp]),
            "h1bkv_import_tokens": (C.c_int, [vp, i32, i32, i32, i32, vp, vp, vp, vp]),
            "h1bkv_extend_seq": (C.c_int, [vp, i32, i32, vp]),
            "h1bkv_profile_enable": (C.c_int, [vp, i32, C.c_uint32]),
            "h1bkv_profile_stride": (C.c_int, [vp, i32]),
            "h1bkv_profile_read": (C.c_int, [vp, i32, vp, i32, C.POINTER(i32)]),
            "h1bkv_stream_copy": (C.c_int, [vp, vp, sz, vp]),
            "h1bkv_stream_read": (C.c_int, [vp, sz, vp, vp]),
            "h1bkv_stream_read_ms": (C.c_int, [vp, sz, vp, vp, C.POINTER(C.c_float)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _ids(seq_ids: Sequence[int]):
    a = np.ascontiguousarray(seq_ids, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dev_ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or a raw integer address / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def h1bkv_version() -> int:
    return lib().h1bkv_version()


def h1bkv_strerror(code: int) -> str:
    return lib().h1bkv_strerror(code).decode()


def h1bkv_pool_bytes(cfg: h1bkv_config) -> int:
    return lib().h1bkv_pool_bytes(C.byref(cfg))


def h1bkv_create(cfg: h1bkv_config, pool, pool_bytes: int, R: Optional[np.ndarray]):
    """Returns (code, handle).  `pool` is a torch uint8 tensor (or None for a bookkeeping-only handle)."""
    Rc = None if R is None else np.ascontiguousarray(R, dtype=np.float32)
    h = C.c_void_p()
    rc = lib().h1bkv_create(C.byref(cfg), _dev_ptr(pool), pool_bytes, _np_ptr(Rc), C.byref(h))
    return rc, h


def h1bkv_destroy(h) -> int:
    return lib().h1bkv_destroy(h)


def h1bkv_get_projection(h, b: int, d: int):
    out = np.empty((b, d), dtype=np.float32)
    return lib().h1bkv_get_projection(h, _np_ptr(out)), out


def h1bkv_seq_len(h, seq_id: int):
    n = C.c_int32(-1)
    return lib().h1bkv_seq_len(h, seq_id, C.byref(n)), n.value


def h1bkv_free_pages(h):
    n = C.c_int32(-1)
    return lib().h1bkv_free_pages(h, C.byref(n)), n.value


def h1bkv_reset_seq(h, seq_id: int) -> int:
    return lib().h1bkv_reset_seq(h, seq_id)


def h1bkv_truncate_seq(h, seq_id: int, new_len: int) -> int:
    return lib().h1bkv_truncate_seq(h, seq_id, new_len)


def h1bkv_append_kv(h, seq_ids, n_new: int, k, v, stride_seq: int, stride_tok: int, stride_head: int, stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_append_kv(h, p, len(ids), n_new, _dev_ptr(k), _dev_ptr(v), stride_seq, stride_tok, stride_head,
                                 _stream(stream))


def h1bkv_decode_workspace_bytes(h, n_seqs: int, max_ctx: int) -> int:
    return lib().h1bkv_decode_workspace_bytes(h, n_seqs, max_ctx)


def h1bkv_decode_attn(h, seq_ids, q, tau: float, out, workspace, workspace_bytes: int, stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_decode_attn(h, p, len(ids), _dev_ptr(q), tau, _dev_ptr(out), _dev_ptr(workspace), workspace_bytes,
                                   _stream(stream))


def h1bkv_decode_attn_static(h, seq_ids, q, tau: float, out, stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_decode_attn_static(h, p, len(ids), _dev_ptr(q), tau, _dev_ptr(out), _stream(stream))


def h1bkv_decode_step(h, seq_ids, k, v, stride_seq: int, stride_head: int, q, tau: float, out, workspace, workspace_bytes: int,
                      stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_decode_step(h, p, len(ids), _dev_ptr(k), _dev_ptr(v), stride_seq, stride_head, _dev_ptr(q), tau,
                                   _dev_ptr(out), _dev_ptr(workspace), workspace_bytes, _stream(stream))


def h1bkv_reserve_seq(h, seq_id: int, n_tokens: int, stream=0) -> int:
    return lib().h1bkv_reserve_seq(h, seq_id, n_tokens, _stream(stream))


def h1bkv_reserved_tokens(h, seq_id: int):
    n = C.c_int32(0)
    rc = lib().h1bkv_reserved_tokens(h, seq_id, C.byref(n))
    return rc, n.value


def h1bkv_decode_step_dev(h, seq_ids, k, v, stride_seq: int, stride_head: int, q, tau: float, out, pos_dev, max_pos: int,
                          workspace, workspace_bytes: int, stream=0, advance: int = 1) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_decode_step_dev(h, p, len(ids), _dev_ptr(k), _dev_ptr(v), stride_seq, stride_head, _dev_ptr(q), tau,
                                       _dev_ptr(out), _dev_ptr(pos_dev), max_pos, advance, _dev_ptr(workspace),
                                       workspace_bytes, _stream(stream))


def h1bkv_set_seq_len(h, seq_id: int, new_len: int) -> int:
    return lib().h1bkv_set_seq_len(h, seq_id, new_len)


def h1bkv_decode_dtau_workspace_bytes(h, n_seqs: int, max_ctx: int) -> int:
    return lib().h1bkv_decode_dtau_workspace_bytes(h, n_seqs, max_ctx)


def h1bkv_decode_attn_dtau(h, seq_ids, q, tau: float, out, dout, workspace, workspace_bytes: int, stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_decode_attn_dtau(h, p, len(ids), _dev_ptr(q), tau, _dev_ptr(out), _dev_ptr(dout), _dev_ptr(workspace),
                                        workspace_bytes, _stream(stream))


def h1bkv_prefill_workspace_bytes(h, n_seqs: int, n_q: int) -> int:
    return lib().h1bkv_prefill_workspace_bytes(h, n_seqs, n_q)


def h1bkv_prefill_attn(h, seq_ids, n_q: int, q, stride_seq: int, stride_tok: int, stride_head: int, tau: float, out, workspace,
                       workspace_bytes: int, stream=0) -> int:
    ids, p = _ids(seq_ids)
    return lib().h1bkv_prefill_attn(h, p, len(ids), n_q, _dev_ptr(q), stride_seq, stride_tok, stride_head, tau, _dev_ptr(out),
                                    _dev_ptr(workspace), workspace_bytes, _stream(stream))


def h1bkv_set_decode_chunk(h, chunk_tokens: int) -> int:
    return lib().h1bkv_set_decode_chunk(h, chunk_tokens)


def h1bkv_set_projection_path(h, use_matrix_cores: int) -> int:
    return lib().h1bkv_set_projection_path(h, use_matrix_cores)


def h1bkv_debug_fail_launch(h, nth: int) -> int:
    return lib().h1bkv_debug_fail_launch(h, nth)


def h1bkv_export_tokens(h, seq_id: int, kv_head: int, t0: int, n: int, W: int, d: int, n_g: int, value_bits: int = 4):
    """Returns (code, sketches [n][W] u64, codes [n][d/2] u8, scale [n][n_g] u16, zero [n][n_g] u16); for a cache
    with fp16 values (value_bits = 16): (code, sketches, values [n][d] u16 fp16 bit patterns, None, None)."""
    sk = np.zeros((n, W), dtype=np.uint64)
    if value_bits == 16:
        vals = np.zeros((n, d), dtype=np.uint16)
        rc = lib().h1bkv_export_tokens(h, seq_id, kv_head, t0, n, _np_ptr(sk), _np_ptr(vals), None, None)
        return rc, sk, vals, None, None
    codes = np.zeros((n, d // 2), dtype=np.uint8)
    scale = np.zeros((n, n_g), dtype=np.uint16)
    zero = np.zeros((n, n_g), dtype=np.uint16)
    rc = lib().h1bkv_export_tokens(h, seq_id, kv_head, t0, n, _np_ptr(sk), _np_ptr(codes), _np_ptr(scale), _np_ptr(zero))
    return rc, sk, codes, scale, zero


def h1bkv_import_tokens(h, seq_id: int, kv_head: int, t0: int, sk, codes, scale, zero) -> int:
    sk = None if sk is None else np.ascontiguousarray(sk, dtype=np.uint64)
    if codes is not None:      # u8 nibble pairs, or u16 fp16 bit patterns for a cache with fp16 values
        codes = np.ascontiguousarray(codes, dtype=np.uint16 if np.asarray(codes).dtype == np.uint16 else np.uint8)
    scale = None if scale is None else np.ascontiguousarray(scale, dtype=np.uint16)
    zero = None if zero is None else np.ascontiguousarray(zero, dtype=np.uint16)
    n = next(a.shape[0] for a in (sk, codes, scale, zero) if a is not None)
    return lib().h1bkv_import_tokens(h, seq_id, kv_head, t0, n, _np_ptr(sk), _np_ptr(codes), _np_ptr(scale), _np_ptr(zero))


def h1bkv_extend_seq(h, seq_id: int, n_new: int, stream=0) -> int:
    return lib().h1bkv_extend_seq(h, seq_id, n_new, _stream(stream))


def h1bkv_profile_enable(h, capacity: int, kernel_mask: int = 0xF) -> int:
    return lib().h1bkv_profile_enable(h, capacity, kernel_mask)


def h1bkv_profile_stride(h, stride: int) -> int:
    return lib().h1bkv_profile_stride(h, stride)


def h1bkv_profile_read(h, kernel: int, cap: int = 4096):
    ms = np.zeros(cap, dtype=np.float32)
    n = C.c_int32(0)
    rc = lib().h1bkv_profile_read(h, kernel, _np_ptr(ms), cap, C.byref(n))
    return rc, ms[: n.value].copy()


def h1bkv_stream_copy(dst, src, n_bytes: int, stream=0) -> int:
    return lib().h1bkv_stream_copy(_dev_ptr(dst), _dev_ptr(src), n_bytes, _stream(stream))


def h1bkv_stream_read(src, n_bytes: int, sink, stream=0) -> int:
    return lib().h1bkv_stream_read(_dev_ptr(src), n_bytes, _dev_ptr(sink), _stream(stream))


def h1bkv_stream_read_ms(src, n_bytes: int, sink, stream=0):
    ms = C.c_float(0.0)
    rc = lib().h1bkv_stream_read_ms(_dev_ptr(src), n_bytes, _dev_ptr(sink), _stream(stream), C.byref(ms))
    return rc, ms.value


def check(code: int, what: str = "h1bkv") -> None:
    if code != H1BKV_OK:
        raise H1BKVError(code, what)


class Cache:
    """Convenience owner of a handle plus the torch buffers it needs.  Forwards to the functions above."""

    def __init__(self, *, n_q_heads: int, n_kv_heads: int, head_dim: int, sketch_bits: int, group_size: int, dtype: str,
                 max_seqs: int, max_pages: int, max_pages_per_seq: int, R: Optional[np.ndarray], device: int = 0,
                 value_bits: int = 4, pool_fill: Optional[int] = None, seed: int = 0):
        """pool_fill: byte value written over the whole pool before the handle is created (never-written slots then hold
        that pattern instead of whatever the allocator returned)."""
        self.cfg = h1bkv_config(n_q_heads, n_kv_heads, head_dim, sketch_bits, group_size,
                                H1BKV_F16 if dtype == "f16" else H1BKV_F32, 0, max_seqs, max_pages, max_pages_per_seq, device,
                                value_bits, seed)
        self.value_bits = value_bits
        self.W, self.d, self.n_g = sketch_bits // 64, head_dim, head_dim // group_size
        self.pool = None
        self.workspace = None
        nbytes = h1bkv_pool_bytes(self.cfg)
        if nbytes == 0:
            raise H1BKVError(H1BKV_ESHAPE, "h1bkv_pool_bytes")
        if device != H1BKV_DEVICE_NONE:
            import torch
            torch.cuda.set_device(device)
            self.pool = torch.empty(nbytes, dtype=torch.uint8, device=f"cuda:{device}")
            if pool_fill is not None:
                self.pool.fill_(pool_fill)
                torch.cuda.synchronize()
        rc, self.h = h1bkv_create(self.cfg, self.pool, nbytes, R)
        check(rc, "h1bkv_create")

    def close(self):
        if getattr(self, "h", None):
            h1bkv_destroy(self.h)
            self.h = None

    def __del__(self):
        # at interpreter shutdown the module's globals may already be gone: the handle then dies with the process
        if h1bkv_destroy is not None:
            self.close()

    def seq_len(self, seq_id: int) -> int:
        rc, n = h1bkv_seq_len(self.h, seq_id)
        check(rc, "h1bkv_seq_len")
        return n

    def append(self, seq_ids, k, v, stream=None) -> None:
        """k, v: torch tensors [n_seqs][n_new][H_kv][d] (any strides with a dense last axis)."""
        assert k.shape == v.shape and k.stride() == v.stride() and k.stride(3) == 1
        check(h1bkv_append_kv(self.h, seq_ids, k.shape[1], k, v, k.stride(0), k.stride(1), k.stride(2), stream), "h1bkv_append_kv")

    def decode(self, seq_ids, q, tau: float, out=None, stream=None):
        import torch
        n = len(seq_ids)
        max_ctx = max(self.seq_len(s) for s in seq_ids)
        need = h1bkv_decode_workspace_bytes(self.h, n, max_ctx)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if out is None:
            out = torch.empty((n, self.cfg.n_q_heads, self.d), dtype=torch.float32, device=q.device)
        check(h1bkv_decode_attn(self.h, seq_ids, q, tau, out, self.workspace, self.workspace.numel(), stream), "h1bkv_decode_attn")
        return out

    def decode_dtau(self, seq_ids, q, tau: float, stream=None):
        """Returns (out, d out / d tau), each [n_seqs][H_q][d] float32."""
        import torch
        n = len(seq_ids)
        max_ctx = max(self.seq_len(s) for s in seq_ids)
        need = h1bkv_decode_dtau_workspace_bytes(self.h, n, max_ctx)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        out = torch.empty((n, self.cfg.n_q_heads, self.d), dtype=torch.float32, device=q.device)
        dout = torch.empty_like(out)
        check(h1bkv_decode_attn_dtau(self.h, seq_ids, q, tau, out, dout, self.workspace, self.workspace.numel(), stream),
              "h1bkv_decode_attn_dtau")
        return out, dout

    def prefill(self, seq_ids, q, tau: float, out=None, stream=None):
        """q: torch tensor [n_seqs][n_q][H_q][d] (dense last axis): the last n_q cached positions attend causally."""
        import torch
        n, n_q = len(seq_ids), q.shape[1]
        need = h1bkv_prefill_workspace_bytes(self.h, n, n_q)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if out is None:
            out = torch.empty((n, n_q, self.cfg.n_q_heads, self.d), dtype=torch.float32, device=q.device)
        assert q.stride(3) == 1
        check(h1bkv_prefill_attn(self.h, seq_ids, n_q, q, q.stride(0), q.stride(1), q.stride(2), tau, out, self.workspace,
                                 self.workspace.numel(), stream), "h1bkv_prefill_attn")
        return out

    def export(self, seq_id: int, kv_head: int, t0: int, n: int):
        rc, sk, codes, scale, zero = h1bkv_export_tokens(self.h, seq_id, kv_head, t0, n, self.W, self.d, self.n_g, self.value_bits)
        check(rc, "h1bkv_export_tokens")
        return sk, codes, scale, zero
