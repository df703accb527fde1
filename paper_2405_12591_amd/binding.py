"""ctypes binding of libdecoquant.so; names follow include/decoquant.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional

import torch

from . import build as _build

DECODE_AUTO = 0
ABI_VERSION = 6   # dq_version() of the library whose struct layouts this file mirrors
COMPRESS_NO_LARGE = 1
COMPRESS_PLAIN = 2
DECODE_FORCE_GENERIC = 1
DECODE_FORCE_MFMA = 2


def decode_flags(kernel: int = DECODE_AUTO, splits: int = 0, waves: int = 0, unit_map: Optional[int] = None) -> int:
    """The flags word of dq_attn_decode: kernel choice plus the launch-shape overrides
    DQ_DECODE_SPLITS / DQ_DECODE_WAVES / DQ_DECODE_UNIT_MAP (0 / None: the library's choice)."""
    return kernel | ((splits & 0x7F) << 8) | ((waves & 0xF) << 16) | (0 if unit_map is None else ((unit_map + 1) & 0xF) << 20)


def compress_flags(keep_large: bool = True, waves: int = 0, plain: bool = False) -> int:
    """The flags word of dq_compress_kv_ex (DQ_COMPRESS_NO_LARGE, DQ_COMPRESS_PLAIN, DQ_COMPRESS_WAVES)."""
    return (0 if keep_large else COMPRESS_NO_LARGE) | (COMPRESS_PLAIN if plain else 0) | ((waves & 0xF) << 8)

EXPORTED_SYMBOLS = [
    "dq_version", "dq_status_string", "dq_last_hip_error", "dq_decode_mfma_supported",
    "dq_decode_workspace_bytes", "dq_workspace_init", "dq_attn_decode", "dq_attn_decode_timed", "dq_attn_decode_tail",
    "dq_attn_decode_static",
    "dq_compress_workspace_bytes", "dq_compress_kv", "dq_compress_blocks_workspace_bytes", "dq_compress_kv_blocks",
    "dq_compress_kv_ex", "dq_cache_append_workspace_bytes", "dq_cache_append",
    "dq_quantize_pack", "dq_stream_read",
]


class DQError(RuntimeError):
    pass


class _CFormat(C.Structure):
    _fields_ = [("bits", C.c_int32), ("group", C.c_int32), ("head_dim", C.c_int32),
                ("j1", C.c_int32), ("j2", C.c_int32), ("block_tokens", C.c_int32), ("i3", C.c_int32),
                ("levels", C.c_int32), ("i1", C.c_int32)]


class _CTail(C.Structure):
    _fields_ = [("k_tail", C.c_void_p), ("v_tail", C.c_void_p), ("tail_lens", C.c_void_p), ("capacity", C.c_int32)]


class _CCache(C.Structure):
    _fields_ = [("k_codes", C.c_void_p), ("k_scales", C.c_void_p), ("k_small", C.c_void_p),
                ("v_codes", C.c_void_p), ("v_scales", C.c_void_p), ("v_small", C.c_void_p),
                ("k_small3", C.c_void_p), ("v_small3", C.c_void_p),
                ("batch", C.c_int32), ("kv_heads", C.c_int32), ("block_capacity", C.c_int32)]


def _load() -> C.CDLL:
    path = os.environ.get("DQ_LIBRARY_PATH") or _build.LIB_PATH   # an alternative build, for experiments
    if path == _build.LIB_PATH and not os.path.exists(path):
        _build.build_library()
    if not os.path.exists(path):
        raise DQError("libdecoquant.so is missing and could not be built")
    l = C.CDLL(path)
    l.dq_version.restype = C.c_int32
    if int(l.dq_version()) != ABI_VERSION:   # the structs below would not match the library's
        raise DQError("%s is version %d, this binding needs %d: rebuild it" % (path, int(l.dq_version()), ABI_VERSION))
    l.dq_status_string.restype = C.c_char_p
    l.dq_status_string.argtypes = [C.c_int32]
    l.dq_last_hip_error.restype = C.c_int32
    l.dq_decode_mfma_supported.restype = C.c_int32
    l.dq_decode_mfma_supported.argtypes = [C.POINTER(_CFormat), C.c_int32, C.c_int32]
    l.dq_decode_workspace_bytes.restype = C.c_size_t
    l.dq_decode_workspace_bytes.argtypes = [C.POINTER(_CFormat), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    l.dq_workspace_init.restype = C.c_int32
    l.dq_workspace_init.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
    l.dq_attn_decode.restype = C.c_int32
    l.dq_attn_decode.argtypes = [C.POINTER(_CFormat), C.POINTER(_CCache), C.c_void_p, C.c_int32, C.c_void_p,
                                 C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                 C.c_uint32, C.c_void_p]
    l.dq_attn_decode_timed.restype = C.c_int32
    l.dq_attn_decode_timed.argtypes = l.dq_attn_decode.argtypes + [C.c_void_p, C.c_void_p]
    l.dq_attn_decode_tail.restype = C.c_int32
    l.dq_attn_decode_tail.argtypes = [C.POINTER(_CFormat), C.POINTER(_CCache), C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int32, C.POINTER(_CTail), C.c_float, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
    l.dq_attn_decode_static.restype = C.c_int32
    l.dq_attn_decode_static.argtypes = [C.POINTER(_CFormat), C.POINTER(_CCache), C.c_void_p, C.c_int32, C.c_void_p,
                                        C.c_int32, C.POINTER(_CTail), C.c_float, C.c_void_p, C.c_void_p,
                                        C.c_uint32, C.c_void_p]
    l.dq_compress_workspace_bytes.restype = C.c_size_t
    l.dq_compress_workspace_bytes.argtypes = [C.POINTER(_CFormat), C.c_int32, C.c_int32]
    l.dq_compress_kv.restype = C.c_int32
    l.dq_compress_kv.argtypes = [C.POINTER(_CFormat), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int32,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    l.dq_compress_blocks_workspace_bytes.restype = C.c_size_t
    l.dq_compress_blocks_workspace_bytes.argtypes = [C.POINTER(_CFormat), C.c_int32, C.c_int32, C.c_int32]
    l.dq_compress_kv_blocks.restype = C.c_int32
    l.dq_compress_kv_blocks.argtypes = l.dq_compress_kv.argtypes
    l.dq_compress_kv_ex.restype = C.c_int32
    l.dq_compress_kv_ex.argtypes = l.dq_compress_kv.argtypes[:-1] + [C.c_uint32, C.c_void_p]
    l.dq_cache_append_workspace_bytes.restype = C.c_size_t
    l.dq_cache_append_workspace_bytes.argtypes = [C.POINTER(_CFormat), C.c_int32, C.c_int32]
    l.dq_cache_append.restype = C.c_int32
    l.dq_cache_append.argtypes = [C.POINTER(_CFormat), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
    l.dq_quantize_pack.restype = C.c_int32
    l.dq_quantize_pack.argtypes = [C.POINTER(_CFormat), C.c_void_p, C.c_int64, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p]
    l.dq_stream_read.restype = C.c_int32
    l.dq_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    return l


lib = _load()


def version() -> int:
    return int(lib.dq_version())


def status_string(status: int) -> str:
    return lib.dq_status_string(status).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        extra = ""
        if status == -3:
            extra = " (hipError %d)" % lib.dq_last_hip_error()
        raise DQError("%s failed: %s%s" % (what, status_string(status), extra))


@dataclass(frozen=True)
class Format:
    bits: int
    group: int
    head_dim: int
    j1: int
    j2: int
    block_tokens: int
    i3: int = 1   # 8: three local tensors (T_3 is 8 x 8 on the token side)
    levels: int = 0   # 1: the quantizer uses all 2^bits codes (not the paper's symmetric range)
    i1: int = 1   # 2 or 4: a token factor on the small tensor, which is then (i1*j1) x (i1*j1)

    def c(self) -> _CFormat:
        return _CFormat(self.bits, self.group, self.head_dim, self.j1, self.j2, self.block_tokens, self.i3,
                        self.levels, self.i1)

    @property
    def small_side(self) -> int:
        return self.i1 * self.j1

    @property
    def row_bytes(self) -> int:
        return self.head_dim * self.bits // 8

    @property
    def groups(self) -> int:
        return self.head_dim // self.group


class Cache:
    """Device tensors of a compressed cache plus the C struct that points at them."""

    def __init__(self, fmt: Format, tensors: Dict[str, torch.Tensor], batch: int, kv_heads: int,
                 block_capacity: int):
        self.fmt, self.t = fmt, tensors
        self.batch, self.kv_heads, self.block_capacity = batch, kv_heads, block_capacity
        for name, ten in tensors.items():
            if not (ten.is_cuda and ten.is_contiguous()):
                raise DQError("cache tensor %s must be a contiguous device tensor" % name)
        for name, (shape, dtype) in _shapes(fmt, batch, kv_heads, block_capacity).items():
            if name not in tensors or tuple(tensors[name].shape) != tuple(shape) or tensors[name].dtype != dtype:
                raise DQError("cache tensor %s must be %s of shape %s" % (name, dtype, tuple(shape)))
        small3 = [tensors[n].data_ptr() if n in tensors else None for n in ("k_small3", "v_small3")]
        self.c = _CCache(*(tensors[n].data_ptr() for n in
                           ("k_codes", "k_scales", "k_small", "v_codes", "v_scales", "v_small")),
                         *small3, batch, kv_heads, block_capacity)

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in self.t.values())

    def clone(self) -> "Cache":
        return Cache(self.fmt, {k: v.clone() for k, v in self.t.items()}, self.batch, self.kv_heads,
                     self.block_capacity)


def _shapes(fmt: Format, b: int, h: int, nb: int):
    tiles = fmt.block_tokens // 128
    extra = {}
    if fmt.i3 > 1:
        extra = {"k_small3": ((b, h, nb, fmt.i3, fmt.i3), torch.float16),
                 "v_small3": ((b, h, nb, fmt.i3, fmt.i3), torch.float16)}
    return {
        **extra,
        "k_codes": ((b, h, nb, fmt.block_tokens, fmt.row_bytes), torch.uint8),
        "k_scales": ((b, h, nb, fmt.block_tokens, fmt.groups), torch.float16),
        "k_small": ((b, h, nb, fmt.small_side, fmt.small_side), torch.float16),
        "v_codes": ((b, h, nb, tiles, fmt.j2, fmt.j1, 128 * fmt.bits // 8), torch.uint8),
        "v_scales": ((b, h, nb, fmt.block_tokens, fmt.groups), torch.float16),
        "v_small": ((b, h, nb, fmt.small_side, fmt.small_side), torch.float16),
    }


def alloc_cache(fmt: Format, batch: int, kv_heads: int, block_capacity: int, device="cuda:0",
                fill: Optional[int] = 0) -> Cache:
    """Allocate the cache arrays.  fill=None leaves them uninitialised."""
    tensors = {}
    for name, (shape, dtype) in _shapes(fmt, batch, kv_heads, block_capacity).items():
        t = torch.empty(shape, dtype=dtype, device=device)
        if fill is not None:
            t.view(torch.uint8).fill_(fill)
        tensors[name] = t
    return Cache(fmt, tensors, batch, kv_heads, block_capacity)


def cache_from_numpy(fmt: Format, arrays, device="cuda:0") -> Cache:
    """Upload host arrays that already follow the storage layout."""
    b, h, nb = arrays["k_codes"].shape[:3]
    tensors = {}
    for name, (shape, dtype) in _shapes(fmt, b, h, nb).items():
        a = arrays[name]
        if tuple(a.shape) != tuple(shape):
            raise DQError("array %s has shape %s, expected %s" % (name, a.shape, shape))
        tensors[name] = torch.from_numpy(a).to(device).contiguous()
        if tensors[name].dtype != dtype:
            raise DQError("array %s has dtype %s" % (name, a.dtype))
    return Cache(fmt, tensors, b, h, nb)


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def decode_workspace(fmt: Format, batch: int, q_heads: int, kv_heads: int, max_seq_len: int,
                     device="cuda:0") -> torch.Tensor:
    cf = fmt.c()
    n = lib.dq_decode_workspace_bytes(C.byref(cf), batch, q_heads, kv_heads, max_seq_len)
    if n == 0:
        raise DQError("dq_decode_workspace_bytes rejected the arguments")
    n = (n + 15) // 16 * 16
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    workspace_init(ws)
    return ws


def compress_workspace(fmt: Format, batch: int, kv_heads: int, device="cuda:0",
                       t_new: Optional[int] = None) -> torch.Tensor:
    """Workspace of compress_kv; with t_new, of compress_kv_blocks for that many rows per sequence."""
    cf = fmt.c()
    if t_new is None:
        n = lib.dq_compress_workspace_bytes(C.byref(cf), batch, kv_heads)
    else:
        n = lib.dq_compress_blocks_workspace_bytes(C.byref(cf), batch, kv_heads, t_new)
    if n == 0:
        raise DQError("the compression workspace query rejected the arguments")
    ws = torch.empty((n + 15) // 16 * 16, dtype=torch.uint8, device=device)
    ws[:256].zero_()   # status words and the counter the no-hand-off path of compress_kv keeps there
    return ws


def workspace_init(ws: torch.Tensor) -> None:
    _check(lib.dq_workspace_init(ws.data_ptr(), ws.numel(), _stream_ptr(ws.device)), "dq_workspace_init")


def attn_decode(cache: Cache, q: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                workspace: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                out_f32: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                flags: int = DECODE_AUTO, kernel_events=None, tail=None) -> torch.Tensor:
    # workspace=None: dq_attn_decode_static (the library's built-in scratch memory, batch * q_heads <= 512)
    """out[b, h_q] = softmax(q . K_hat^T * scale) V_hat over the compressed cache (dq_attn_decode).

    kernel_events: optional (start, stop) torch.cuda.Event pair, each already recorded once so
    that its handle exists; they are re-recorded around the main kernel (dq_attn_decode_timed).
    tail: optional (k_tail, v_tail, tail_lens) fp16 [B, H_kv, cap, d] + int32 [B]: the tokens not
    yet compressed (dq_attn_decode_tail).
    """
    fmt = cache.fmt
    if q.dtype != torch.float16 or not q.is_contiguous() or seq_lens.dtype != torch.int32:
        raise DQError("q must be contiguous fp16 and seq_lens int32")
    # the library sees pointers only: sizes are checked here, so that a tensor of the wrong shape
    # raises instead of sending a kernel past its end
    if q.dim() != 3 or q.shape[0] != cache.batch or q.shape[2] != fmt.head_dim:
        raise DQError("q must be [batch, q_heads, head_dim] with the cache's batch and head_dim")
    bsz, hq, d = q.shape
    if seq_lens.numel() != bsz or not seq_lens.is_contiguous():
        raise DQError("seq_lens must hold one length per sequence")
    if out is None:
        out = torch.empty_like(q)
    elif out.shape != q.shape or out.dtype != torch.float16 or not out.is_contiguous():
        raise DQError("out must be contiguous fp16 of q's shape")
    if out_f32 is not None and (out_f32.shape != q.shape or out_f32.dtype != torch.float32 or not out_f32.is_contiguous()):
        raise DQError("out_f32 must be contiguous fp32 of q's shape")
    cf = fmt.c()
    ct = None
    if tail is not None:
        ct = _tail_struct(cache, tail, bsz)
    if workspace is None:
        if kernel_events is not None:
            raise DQError("kernel events need a workspace call")
        st = lib.dq_attn_decode_static(C.byref(cf), C.byref(cache.c), q.data_ptr(), hq, seq_lens.data_ptr(), max_seq_len,
                                       None if ct is None else C.byref(ct), softmax_scale, out.data_ptr(),
                                       0 if out_f32 is None else out_f32.data_ptr(), flags, _stream_ptr(q.device))
        _check(st, "dq_attn_decode_static")
        return out
    args = (C.byref(cf), C.byref(cache.c), q.data_ptr(), hq, seq_lens.data_ptr(), max_seq_len,
            softmax_scale, out.data_ptr(), 0 if out_f32 is None else out_f32.data_ptr(),
            workspace.data_ptr(), workspace.numel(), flags, _stream_ptr(q.device))
    if tail is not None:
        st = lib.dq_attn_decode_tail(*args[:6], C.byref(ct), *args[6:])
    elif kernel_events is None:
        st = lib.dq_attn_decode(*args)
    else:
        st = lib.dq_attn_decode_timed(*args, kernel_events[0].cuda_event, kernel_events[1].cuda_event)
    _check(st, "dq_attn_decode")
    return out


def _tail_struct(cache: Cache, tail, bsz: int) -> _CTail:
    kt, vt, tl = tail
    if kt.dtype != torch.float16 or vt.dtype != torch.float16 or tl.dtype != torch.int32 \
            or not kt.is_contiguous() or not vt.is_contiguous():
        raise DQError("tail tensors must be contiguous fp16 with int32 lengths")
    if kt.dim() != 4 or kt.shape != vt.shape or kt.shape[0] != bsz or kt.shape[1] != cache.kv_heads \
            or kt.shape[3] != cache.fmt.head_dim or tl.numel() != bsz or not tl.is_contiguous():
        raise DQError("tail tensors must be [batch, kv_heads, capacity, head_dim] with one length per sequence")
    return _CTail(kt.data_ptr(), vt.data_ptr(), tl.data_ptr(), kt.shape[2])


def _check_compress_args(cache: Cache, k_new, v_new, blk_idx, n_valid) -> None:
    # sizes are checked here (the library sees pointers only)
    for t in (k_new, v_new):
        if t.dtype != torch.float16 or not t.is_contiguous():
            raise DQError("k_new/v_new must be contiguous fp16")
    if k_new.dim() != 4 or k_new.shape != v_new.shape or k_new.shape[0] != cache.batch \
            or k_new.shape[1] != cache.kv_heads or k_new.shape[3] != cache.fmt.head_dim:
        raise DQError("k_new/v_new must be [batch, kv_heads, t_new, head_dim] of the cache's sizes")
    for name, t in (("blk_idx", blk_idx), ("n_valid", n_valid)):
        if t is not None and (t.dtype != torch.int32 or t.numel() != cache.batch or not t.is_contiguous()):
            raise DQError("%s must hold one int32 per sequence" % name)


def compress_kv(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, blk_idx: torch.Tensor,
                n_valid: Optional[torch.Tensor], workspace: torch.Tensor, keep_large: bool = True,
                waves: int = 0, plain: bool = False) -> None:
    """Compress k_new, v_new [B, H, t_new, d] into block slot blk_idx[b] (dq_compress_kv).
    keep_large=False: the fp32 large tensors need not be left in the workspace
    (dq_compress_kv_ex with DQ_COMPRESS_NO_LARGE); waves, plain: its launch overrides."""
    _check_compress_args(cache, k_new, v_new, blk_idx, n_valid)
    fmt_c = cache.fmt.c()
    t_new = k_new.shape[2]
    if t_new > cache.fmt.block_tokens:
        raise DQError("compress_kv takes at most one block of rows; compress_kv_blocks takes more")
    args = (C.byref(fmt_c), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(), t_new,
            blk_idx.data_ptr(), 0 if n_valid is None else n_valid.data_ptr(),
            workspace.data_ptr(), workspace.numel())
    if keep_large and not waves and not plain:
        _check(lib.dq_compress_kv(*args, _stream_ptr(k_new.device)), "dq_compress_kv")
    else:
        _check(lib.dq_compress_kv_ex(*args, compress_flags(keep_large, waves, plain), _stream_ptr(k_new.device)),
               "dq_compress_kv_ex")


def compress_kv_blocks(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, blk_idx: torch.Tensor,
                       n_valid: Optional[torch.Tensor], workspace: torch.Tensor, keep_large: bool = True,
                       waves: int = 0, plain: bool = False) -> None:
    """Compress k_new, v_new [B, H, t_new, d], any t_new >= 1, into the block slots from blk_idx[b]
    on (dq_compress_kv_blocks; dq_compress_kv_ex when a flag is given)."""
    _check_compress_args(cache, k_new, v_new, blk_idx, n_valid)
    cf = cache.fmt.c()
    args = (C.byref(cf), C.byref(cache.c), k_new.data_ptr(), v_new.data_ptr(),
            k_new.shape[2], blk_idx.data_ptr(), 0 if n_valid is None else n_valid.data_ptr(),
            workspace.data_ptr(), workspace.numel())
    if keep_large and not waves and not plain:
        _check(lib.dq_compress_kv_blocks(*args, _stream_ptr(k_new.device)), "dq_compress_kv_blocks")
    else:
        _check(lib.dq_compress_kv_ex(*args, compress_flags(keep_large, waves, plain), _stream_ptr(k_new.device)),
               "dq_compress_kv_ex")


def quantize_pack(fmt: Format, t_large: torch.Tensor, value_layout: bool):
    """Quantize + pack fp32 rows [n_rows, d]; returns (codes u8, scales f16) (dq_quantize_pack)."""
    if t_large.dtype != torch.float32 or not t_large.is_contiguous():
        raise DQError("t_large must be contiguous fp32")
    if t_large.dim() != 2 or t_large.shape[1] != fmt.head_dim or t_large.shape[0] % 128:
        raise DQError("t_large must be [n_rows, head_dim] with n_rows a multiple of 128")
    n_rows, d = t_large.shape
    if value_layout:
        codes = torch.empty((n_rows // 128, fmt.j2, fmt.j1, 128 * fmt.bits // 8), dtype=torch.uint8,
                            device=t_large.device)
    else:
        codes = torch.empty((n_rows, fmt.row_bytes), dtype=torch.uint8, device=t_large.device)
    scales = torch.empty((n_rows, fmt.groups), dtype=torch.float16, device=t_large.device)
    cf = fmt.c()
    st = lib.dq_quantize_pack(C.byref(cf), t_large.data_ptr(), n_rows, 1 if value_layout else 0,
                              codes.data_ptr(), scales.data_ptr(), _stream_ptr(t_large.device))
    _check(st, "dq_quantize_pack")
    return codes, scales


def stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib.dq_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(src.device)), "dq_stream_read")


def decode_mfma_supported(fmt: Format, q_heads: int, kv_heads: int) -> bool:
    cf = fmt.c()
    return bool(lib.dq_decode_mfma_supported(C.byref(cf), q_heads, kv_heads))


class _CKVState(C.Structure):
    _fields_ = [("k_tail", C.c_void_p), ("v_tail", C.c_void_p), ("tail_lens", C.c_void_p), ("seq_lens", C.c_void_p)]


APPEND_NO_COMPRESS = 1


def cache_append_workspace(fmt: Format, batch: int, kv_heads: int, device="cuda:0") -> torch.Tensor:
    cf = fmt.c()
    n = lib.dq_cache_append_workspace_bytes(C.byref(cf), batch, kv_heads)
    if n == 0:
        raise DQError("dq_cache_append_workspace_bytes rejected the arguments")
    ws = torch.empty((n + 15) // 16 * 16, dtype=torch.uint8, device=device)
    workspace_init(ws)
    return ws


def cache_append(cache: Cache, k_tail: torch.Tensor, v_tail: torch.Tensor, tail_lens: torch.Tensor,
                 seq_lens: torch.Tensor, k_rows: torch.Tensor, v_rows: torch.Tensor,
                 counts: Optional[torch.Tensor], workspace: torch.Tensor, flags: int = 0) -> None:
    """Append k_rows, v_rows [B, H, n_rows, d] (sequence b takes the first counts[b]) to the fp16
    tails and compress every tail that fills, all decided on the device (dq_cache_append)."""
    fmt = cache.fmt
    want_tail = (cache.batch, cache.kv_heads, fmt.block_tokens, fmt.head_dim)
    for name, t in (("k_tail", k_tail), ("v_tail", v_tail)):
        if t.dtype != torch.float16 or not t.is_contiguous() or tuple(t.shape) != want_tail:
            raise DQError("%s must be contiguous fp16 [batch, kv_heads, block_tokens, head_dim]" % name)
    for name, t in (("tail_lens", tail_lens), ("seq_lens", seq_lens), ("counts", counts)):
        if t is not None and (t.dtype != torch.int32 or t.numel() != cache.batch or not t.is_contiguous()):
            raise DQError("%s must hold one int32 per sequence" % name)
    for t in (k_rows, v_rows):
        if t.dtype != torch.float16 or not t.is_contiguous():
            raise DQError("k_rows/v_rows must be contiguous fp16")
    if k_rows.dim() != 4 or k_rows.shape != v_rows.shape or tuple(k_rows.shape[:2]) != want_tail[:2] \
            or k_rows.shape[3] != fmt.head_dim or not 1 <= k_rows.shape[2] <= fmt.block_tokens:
        raise DQError("k_rows/v_rows must be [batch, kv_heads, n_rows <= block_tokens, head_dim]")
    cf = fmt.c()
    state = _CKVState(k_tail.data_ptr(), v_tail.data_ptr(), tail_lens.data_ptr(), seq_lens.data_ptr())
    st = lib.dq_cache_append(C.byref(cf), C.byref(cache.c), C.byref(state), k_rows.data_ptr(), v_rows.data_ptr(),
                             k_rows.shape[2], 0 if counts is None else counts.data_ptr(), workspace.data_ptr(),
                             workspace.numel(), flags, _stream_ptr(k_rows.device))
    _check(st, "dq_cache_append")


class KVCacheLayer:
    """One layer's KV cache under the paper's policy (Section 3.2): new key/value rows go to an
    fp16 tail; whenever a sequence's tail holds a whole block it is compressed into the next block
    slot; decode attends to the compressed blocks and the tail.  The lengths live on the device and
    every decision is taken there (dq_cache_append); this class only holds the tensors and passes
    pointers.  The one thing the host tracks is an upper bound on the rows any sequence can hold,
    which sizes the decode launch."""

    def __init__(self, fmt: Format, batch: int, q_heads: int, kv_heads: int, max_tokens: int, device="cuda:0"):
        self.fmt, self.batch, self.q_heads, self.kv_heads, self.device = fmt, batch, q_heads, kv_heads, device
        tb = fmt.block_tokens
        self.capacity_blocks = -(-max_tokens // tb)
        self.cache = alloc_cache(fmt, batch, kv_heads, self.capacity_blocks, device)
        self.k_tail = torch.zeros((batch, kv_heads, tb, fmt.head_dim), dtype=torch.float16, device=device)
        self.v_tail = torch.zeros_like(self.k_tail)
        self.seq_lens = torch.zeros(batch, dtype=torch.int32, device=device)    # compressed tokens per sequence
        self.tail_lens = torch.zeros(batch, dtype=torch.int32, device=device)   # rows in the fp16 tail
        self.ws_decode = decode_workspace(fmt, batch, q_heads, kv_heads, self.capacity_blocks * tb, device)
        self.ws_append = cache_append_workspace(fmt, batch, kv_heads, device)
        self._ws_prefill = None
        self.rows_upper = 0                  # no sequence holds more rows than this (host-side bound)

    # ---- the device-side lengths, read back (tests and diagnostics; not used on the step path) ----
    @property
    def n_blocks(self):
        return (self.seq_lens // self.fmt.block_tokens).tolist()

    @property
    def n_tail(self):
        return self.tail_lens.tolist()

    @property
    def status(self) -> int:
        """Bit 0: a tail filled while its sequence had no free block slot (rows were dropped)."""
        return int(self.ws_append[12:16].view(torch.int32).item())

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, counts=None) -> None:
        """Append rows k_new, v_new [B, H_kv, n, d]; sequence b takes the first counts[b] rows
        (counts: int32 device tensor, a list, or None for all n).  Full tails are compressed on the way."""
        tb = self.fmt.block_tokens
        n = k_new.shape[2]
        if counts is not None and not torch.is_tensor(counts):
            counts = torch.tensor(list(counts), dtype=torch.int32, device=self.device)
        for lo in range(0, n, tb):           # at most one block's worth of rows per call
            hi = min(n, lo + tb)
            kr, vr = k_new[:, :, lo:hi], v_new[:, :, lo:hi]
            if not kr.is_contiguous():
                kr, vr = kr.contiguous(), vr.contiguous()
            c = None if counts is None else torch.clamp(counts - lo, 0, hi - lo).to(torch.int32)
            cache_append(self.cache, self.k_tail, self.v_tail, self.tail_lens, self.seq_lens, kr, vr, c, self.ws_append)
        self.rows_upper += n

    def prefill(self, k_new: torch.Tensor, v_new: torch.Tensor, counts=None) -> None:
        """Append the rows of a prompt, k_new, v_new [B, H_kv, n, d], to EMPTY sequences; sequence b
        takes the first counts[b] rows (default: all n).  The whole blocks of all sequences are
        compressed by one dq_compress_kv_ex call, the rest goes to the tails."""
        if self.rows_upper:
            raise DQError("prefill needs empty sequences; use append")
        tb = self.fmt.block_tokens
        n = k_new.shape[2]
        if n // tb > self.capacity_blocks:
            raise DQError("the prompt exceeds the cache capacity")
        if counts is None:
            counts = torch.full((self.batch,), n, dtype=torch.int32, device=self.device)
        elif not torch.is_tensor(counts):
            counts = torch.tensor(list(counts), dtype=torch.int32, device=self.device)
        counts = torch.clamp(counts, 0, n).to(torch.int32)
        whole = (counts // tb) * tb                                     # rows that fill whole blocks
        if n >= tb:
            rows = (n // tb) * tb
            if self._ws_prefill is None or self._ws_prefill[0] != rows:
                self._ws_prefill = (rows, compress_workspace(self.fmt, self.batch, self.kv_heads, self.device, t_new=rows))
            first = torch.where(whole > 0, torch.zeros_like(whole), torch.full_like(whole, -1))
            compress_kv_blocks(self.cache, k_new[:, :, :rows].contiguous(), v_new[:, :, :rows].contiguous(),
                               first, whole, self._ws_prefill[1], keep_large=False)
            self.seq_lens.copy_(whole)
        # what is left of every prompt (fewer than block_tokens rows) goes to the tails
        width = min(tb, n)
        idx = torch.clamp(whole.long()[:, None] + torch.arange(width, device=self.device)[None, :], max=n - 1)
        idx = idx[:, None, :, None].expand(self.batch, self.kv_heads, width, self.fmt.head_dim)
        cache_append(self.cache, self.k_tail, self.v_tail, self.tail_lens, self.seq_lens,
                     torch.gather(k_new, 2, idx).contiguous(), torch.gather(v_new, 2, idx).contiguous(),
                     (counts - whole).to(torch.int32), self.ws_append, flags=APPEND_NO_COMPRESS)   # fewer than a block each
        self.rows_upper = n

    def decode(self, q: torch.Tensor, out: Optional[torch.Tensor] = None, flags: int = DECODE_AUTO,
               max_seq_len: Optional[int] = None) -> torch.Tensor:
        """Attention of one query per (sequence, query head) over blocks and tail.  max_seq_len: host
        bound on the compressed tokens of any sequence (default: from the rows appended so far)."""
        tb = self.fmt.block_tokens
        if max_seq_len is None:
            max_seq_len = min(self.capacity_blocks, self.rows_upper // tb) * tb
        return attn_decode(self.cache, q, self.seq_lens, max_seq_len, self.ws_decode, out=out, flags=flags,
                           tail=(self.k_tail, self.v_tail, self.tail_lens))
