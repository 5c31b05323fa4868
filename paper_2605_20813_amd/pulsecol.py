"""Thin ctypes binding over libpulsecol.so: argument marshalling only.

Function names follow include/pulsecol.h.  PyTorch supplies device memory and the
current HIP stream; every step of the method runs inside the library's kernels.  There is
no fallback: if the shared library is missing, loading raises.
"""

from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpulsecol.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_ALIGNMENT, ERR_NO_PATTERN, ERR_OOM, ERR_HIP, ERR_BAD_INDEX = range(8)
BF16, F32 = 0, 1

EXPORTS = (
    "pulsecol_validate_shape", "pulsecol_create", "pulsecol_destroy", "pulsecol_set_validation", "pulsecol_set_attn_block", "pulsecol_set_seq_lens", "pulsecol_num_keep",
    "pulsecol_select", "pulsecol_scores", "pulsecol_topk", "pulsecol_attn", "pulsecol_attn_dense",
    "pulsecol_attn_block", "pulsecol_num_keep_blocks", "pulsecol_select_blocks",
    "pulsecol_refresh_dense", "pulsecol_select_noalloc",
    "pulsecol_refresh_schedule", "pulsecol_refresh_schedule_power", "pulsecol_refresh_schedule_random",
    "pulsecol_attn_tile_shape", "pulsecol_status_str", "pulsecol_last_error",
)


class Shape(ctypes.Structure):
    _fields_ = [("batch", c_int32), ("heads", c_int32), ("seq", c_int32), ("head_dim", c_int32),
                ("dtype", c_int32), ("group_size", c_int32),
                ("stride_b", c_int64), ("stride_h", c_int64), ("stride_n", c_int64),
                ("scale", c_float), ("kv_heads", c_int32),
                ("kv_stride_b", c_int64), ("kv_stride_h", c_int64), ("kv_stride_n", c_int64),
                ("max_keep_ratio", c_double)]


class PulseColError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pulsecol status {status}: {message}")
        self.status = status


_lib = None
# block size every new Context asks for with one set per head (0 = the library's own choice); the test-suite
# sets it to run the same cases through both kernels
DEFAULT_ATTN_BLOCK = 0


def lib() -> ctypes.CDLL:
    """Load libpulsecol.so (built by ``python -m paper_2605_20813_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_20813_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.pulsecol_validate_shape.argtypes = [POINTER(Shape)]
        L.pulsecol_create.argtypes = [POINTER(c_void_p), POINTER(Shape), c_int]
        L.pulsecol_destroy.argtypes = [c_void_p]
        L.pulsecol_set_validation.argtypes = [c_void_p, c_int]
        L.pulsecol_set_attn_block.argtypes = [c_void_p, c_int32]
        L.pulsecol_set_seq_lens.argtypes = [c_void_p, POINTER(c_int32), c_void_p]
        L.pulsecol_num_keep.argtypes = [c_int32, c_double]
        L.pulsecol_num_keep.restype = c_int32
        L.pulsecol_select.argtypes = [c_void_p, c_void_p, c_void_p, c_double, c_int, c_void_p, c_void_p]
        L.pulsecol_scores.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.pulsecol_topk.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
        L.pulsecol_attn.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
        L.pulsecol_attn_dense.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.pulsecol_attn_block.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
        L.pulsecol_num_keep_blocks.argtypes = [c_int32, c_double]
        L.pulsecol_num_keep_blocks.restype = c_int32
        L.pulsecol_select_blocks.argtypes = [c_void_p, c_void_p, c_void_p, c_double, c_void_p, c_void_p]
        L.pulsecol_refresh_dense.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_double, c_void_p, c_void_p, c_void_p]
        L.pulsecol_select_noalloc.argtypes = [POINTER(Shape), c_void_p, c_void_p, c_double, c_void_p, c_void_p]
        L.pulsecol_refresh_schedule.argtypes = [c_int32, c_double, c_int32, POINTER(c_int32)]
        L.pulsecol_refresh_schedule.restype = c_int32
        L.pulsecol_refresh_schedule_power.argtypes = [c_int32, c_double, c_int32, POINTER(c_int32)]
        L.pulsecol_refresh_schedule_power.restype = c_int32
        L.pulsecol_refresh_schedule_random.argtypes = [c_int32, c_double, c_int32, POINTER(c_double), POINTER(c_int32)]
        L.pulsecol_refresh_schedule_random.restype = c_int32
        L.pulsecol_attn_tile_shape.argtypes = [c_void_p, c_int32, POINTER(c_int32), POINTER(c_int32)]
        L.pulsecol_status_str.argtypes = [c_int]
        L.pulsecol_status_str.restype = c_char_p
        L.pulsecol_last_error.argtypes = [c_void_p]
        L.pulsecol_last_error.restype = c_char_p
        _lib = L
    return _lib


def _dtype_code(dtype) -> int:
    if dtype in (torch.bfloat16, "bf16", BF16):
        return BF16
    if dtype in (torch.float32, "f32", F32):
        return F32
    raise ValueError(f"unsupported dtype {dtype}")


def make_shape(batch, heads, seq, head_dim, dtype, group_size=0, strides=(0, 0, 0), scale=0.0,
               kv_heads=0, kv_strides=(0, 0, 0), max_keep_ratio=0.0) -> Shape:
    return Shape(batch, heads, seq, head_dim, _dtype_code(dtype), group_size, *strides, scale, kv_heads, *kv_strides,
                 max_keep_ratio)


def validate_shape(shape: Shape) -> int:
    return lib().pulsecol_validate_shape(ctypes.byref(shape))


def num_keep(seq: int, keep_ratio: float) -> int:
    return lib().pulsecol_num_keep(seq, keep_ratio)


def num_keep_blocks(seq: int, keep_ratio: float) -> int:
    return lib().pulsecol_num_keep_blocks(seq, keep_ratio)


def refresh_schedule(T: int, eta: float, R: int):
    buf = (c_int32 * max(R, 1))()
    r = lib().pulsecol_refresh_schedule(T, eta, R, buf)
    if r < 0:
        raise PulseColError(ERR_INVALID_ARG, "pulsecol_refresh_schedule: bad arguments")
    return list(buf[:r])


def refresh_schedule_power(T: int, eta: float, R: int):
    buf = (c_int32 * max(R, 1))()
    r = lib().pulsecol_refresh_schedule_power(T, eta, R, buf)
    if r < 0:
        raise PulseColError(ERR_INVALID_ARG, "pulsecol_refresh_schedule_power: bad arguments")
    return list(buf[:r])


def refresh_schedule_random(T: int, eta: float, R: int, uniforms):
    u = [float(x) for x in uniforms]
    buf = (c_int32 * max(R, 1))()
    ubuf = (c_double * max(len(u), 1))(*u)
    if len(u) < R - 1:
        raise PulseColError(ERR_INVALID_ARG, "pulsecol_refresh_schedule_random: need R-1 uniforms")
    r = lib().pulsecol_refresh_schedule_random(T, eta, R, ubuf, buf)
    if r < 0:
        raise PulseColError(ERR_INVALID_ARG, "pulsecol_refresh_schedule_random: bad arguments")
    return list(buf[:r])


def status_str(status: int) -> str:
    return lib().pulsecol_status_str(status).decode()


def last_error(handle=None) -> str:
    return lib().pulsecol_last_error(handle).decode()


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def select_noalloc(shape: Shape, Q, K, keep_ratio: float, idx_out):
    """pulsecol_select_noalloc on the current device: the caller brings idx_out [B, H, U, k] (int32)."""
    st = lib().pulsecol_select_noalloc(ctypes.byref(shape), _ptr(Q), _ptr(K), keep_ratio, _ptr(idx_out), _stream())
    if st != OK:
        raise PulseColError(st, last_error(None))
    return idx_out


class Context:
    """Owns one pulsecol_ctx.  Tensors are [B, H, n, d] on the context's device."""

    def __init__(self, batch, heads, seq, head_dim, dtype, group_size=0, strides=(0, 0, 0), scale=0.0, device=0,
                 kv_heads=0, kv_strides=(0, 0, 0), max_keep_ratio=0.0):
        self.shape = make_shape(batch, heads, seq, head_dim, dtype, group_size, strides, scale, kv_heads, kv_strides,
                                max_keep_ratio)
        self.torch_dtype = torch.bfloat16 if self.shape.dtype == BF16 else torch.float32
        self.device = torch.device("cuda", device)
        self._h = c_void_p()
        st = lib().pulsecol_create(ctypes.byref(self._h), ctypes.byref(self.shape), device)
        if st != OK:
            self._h = None
            raise PulseColError(st, last_error(None))
        if DEFAULT_ATTN_BLOCK:
            self.set_attn_block(DEFAULT_ATTN_BLOCK)

    # -- lifetime
    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib().pulsecol_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def _check(self, st):
        if st != OK:
            raise PulseColError(st, last_error(self._h))

    def _check_tensor(self, t, name):
        """Shape and strides of a tensor argument; K and V follow the K/V head count and strides."""
        s = self.shape
        if t.device != self.device or t.dtype != self.torch_dtype:
            raise ValueError(f"{name}: expected {self.torch_dtype} on {self.device}")
        kv = name in ("K", "V")
        kv_follows_q = s.kv_heads in (0, s.heads) and not (s.kv_stride_b or s.kv_stride_h or s.kv_stride_n)
        if kv and not kv_follows_q:
            heads, sb, sh, sn = s.kv_heads or s.heads, s.kv_stride_b, s.kv_stride_h, s.kv_stride_n
        else:
            heads, sb, sh, sn = s.heads, s.stride_b, s.stride_h, s.stride_n
        if tuple(t.shape) != (s.batch, heads, s.seq, s.head_dim):
            raise ValueError(f"{name}: expected shape {(s.batch, heads, s.seq, s.head_dim)}, got {tuple(t.shape)}")
        want = (sb or heads * (sh or s.seq * (sn or s.head_dim)), sh or s.seq * (sn or s.head_dim), sn or s.head_dim, 1)
        if tuple(t.stride()) != want:
            raise ValueError(f"{name}: strides {tuple(t.stride())} do not match the context's {want}")

    def _new_output(self):
        """An O with the context's own strides (a padded row stride makes it larger than a packed tensor)."""
        s = self.shape
        sn = s.stride_n or s.head_dim
        sh = s.stride_h or s.seq * sn
        sb = s.stride_b or s.heads * sh
        return torch.empty_strided((s.batch, s.heads, s.seq, s.head_dim), (sb, sh, sn, 1),
                                   dtype=self.torch_dtype, device=self.device)

    @property
    def groups(self) -> int:
        """U: query groups per head (Sec. 3.3); 1 when the whole head is one group."""
        s = self.shape
        if s.group_size == 0 or s.group_size >= s.seq:
            return 1
        return (s.seq + s.group_size - 1) // s.group_size

    def set_validation(self, on: bool = True):
        """Check column numbers on the device in front of every attn call (synchronises)."""
        self._check(lib().pulsecol_set_validation(self._h, int(bool(on))))

    def set_attn_block(self, block_m: int = 0):
        """Kernel of attn with one set per head: 256 scheduled, 128 plain, 0 the library's choice."""
        self._check(lib().pulsecol_set_attn_block(self._h, int(block_m)))

    def set_seq_lens(self, seq_lens=None):
        """Variable-length batch: per-element lengths (a sequence of `batch` ints), or None for fixed length."""
        if seq_lens is None:
            self._check(lib().pulsecol_set_seq_lens(self._h, None, _stream()))
            return
        lens = [int(x) for x in seq_lens]
        if len(lens) != self.shape.batch:
            raise ValueError("seq_lens: one length per batch element")
        self._check(lib().pulsecol_set_seq_lens(self._h, (c_int32 * len(lens))(*lens), _stream()))

    def tile_shape(self, k: int):
        """(B_M, B_N) of the kernel that attn runs with k kept columns."""
        bm, bn = c_int32(), c_int32()
        self._check(lib().pulsecol_attn_tile_shape(self._h, k, ctypes.byref(bm), ctypes.byref(bn)))
        return bm.value, bn.value

    # -- the calls of include/pulsecol.h
    def select(self, Q, K, keep_ratio: float, refresh: bool = True, idx_out=None):
        s = self.shape
        k = num_keep(s.seq, keep_ratio)
        if k < 0:
            raise PulseColError(ERR_INVALID_ARG, "keep_ratio must be in (0, 1]")
        if idx_out is None:
            idx_out = torch.empty(s.batch, s.heads, self.groups, k, dtype=torch.int32, device=self.device)
        if refresh:
            self._check_tensor(Q, "Q")
            self._check_tensor(K, "K")
        self._check(lib().pulsecol_select(self._h, _ptr(Q) if refresh else None, _ptr(K) if refresh else None,
                                          keep_ratio, int(bool(refresh)), _ptr(idx_out), _stream()))
        return idx_out

    def scores(self, Q, K, scores_out=None):
        s = self.shape
        self._check_tensor(Q, "Q")
        self._check_tensor(K, "K")
        if scores_out is None:
            scores_out = torch.empty(s.batch, s.heads, self.groups, s.seq, dtype=torch.float32, device=self.device)
        self._check(lib().pulsecol_scores(self._h, _ptr(Q), _ptr(K), _ptr(scores_out), _stream()))
        return scores_out

    def topk(self, scores, k: int, idx_out=None):
        s = self.shape
        if scores.dtype != torch.float32 or not scores.is_contiguous() or scores.device != self.device \
                or scores.numel() != s.batch * s.heads * self.groups * s.seq:
            raise ValueError("scores: expected contiguous fp32 [B, H, U, seq] on the context's device")
        if idx_out is None:
            idx_out = torch.empty(s.batch, s.heads, self.groups, max(k, 1), dtype=torch.int32, device=self.device)
        self._check(lib().pulsecol_topk(self._h, _ptr(scores), k, _ptr(idx_out), _stream()))
        return idx_out

    def attn(self, Q, K, V, idx, O=None):
        for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
            self._check_tensor(t, nm)
        s = self.shape
        if idx.dtype != torch.int32 or not idx.is_contiguous() or idx.device != self.device \
                or idx.dim() != 4 or tuple(idx.shape[:3]) != (s.batch, s.heads, self.groups):
            raise ValueError("idx: expected contiguous int32 [B, H, U, k] on the context's device")
        if O is None:
            O = self._new_output()
        self._check_tensor(O, "O")
        self._check(lib().pulsecol_attn(self._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), idx.shape[3], _ptr(O), _stream()))
        return O

    def select_blocks(self, Q, K, keep_ratio: float, block_idx_out=None):
        """Key blocks (of 64 keys) per query block by block mass; returns int32 [B, H, U, kb]."""
        s = self.shape
        kb = num_keep_blocks(s.seq, keep_ratio)
        if kb < 0:
            raise PulseColError(ERR_INVALID_ARG, "need seq % 64 == 0 and keep_ratio in (0, 1]")
        self._check_tensor(Q, "Q")
        self._check_tensor(K, "K")
        if block_idx_out is None:
            block_idx_out = torch.empty(s.batch, s.heads, self.groups, kb, dtype=torch.int32, device=self.device)
        self._check(lib().pulsecol_select_blocks(self._h, _ptr(Q), _ptr(K), keep_ratio, _ptr(block_idx_out), _stream()))
        return block_idx_out

    def attn_block(self, Q, K, V, block_idx, O=None):
        """Block-sparse attention: block_idx int32 [B, H, U, kb] names key blocks of 64 keys."""
        for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
            self._check_tensor(t, nm)
        s = self.shape
        if block_idx.dtype != torch.int32 or not block_idx.is_contiguous() or block_idx.device != self.device \
                or block_idx.dim() != 4 or tuple(block_idx.shape[:3]) != (s.batch, s.heads, self.groups):
            raise ValueError("block_idx: expected contiguous int32 [B, H, U, kb] on the context's device")
        if O is None:
            O = self._new_output()
        self._check_tensor(O, "O")
        self._check(lib().pulsecol_attn_block(self._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(block_idx), block_idx.shape[3],
                                              _ptr(O), _stream()))
        return O

    def refresh_dense(self, Q, K, V, keep_ratio: float, O=None, idx_out=None):
        """Dense output and the new pattern of a refresh step in one call; returns (O, idx)."""
        for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
            self._check_tensor(t, nm)
        s = self.shape
        k = num_keep(s.seq, keep_ratio)
        if k < 0:
            raise PulseColError(ERR_INVALID_ARG, "keep_ratio must be in (0, 1]")
        if O is None:
            O = self._new_output()
        self._check_tensor(O, "O")
        if idx_out is None:
            idx_out = torch.empty(s.batch, s.heads, self.groups, k, dtype=torch.int32, device=self.device)
        self._check(lib().pulsecol_refresh_dense(self._h, _ptr(Q), _ptr(K), _ptr(V), keep_ratio, _ptr(O),
                                                 _ptr(idx_out), _stream()))
        return O, idx_out

    def attn_dense(self, Q, K, V, O=None, lse_out=None):
        for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
            self._check_tensor(t, nm)
        if O is None:
            O = self._new_output()
        self._check_tensor(O, "O")
        self._check(lib().pulsecol_attn_dense(self._h, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(lse_out), _stream()))
        return O
