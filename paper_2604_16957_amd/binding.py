"""ctypes binding of include/tq.h: same names, argument marshalling only.

There is no fallback: if the HIP library has not been built the import of any entry point
fails loudly (build it with `python -m paper_2604_16957_amd.build`).
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libtq_mi355x.so"

TQ_OK = 0
TQ_ERR_NULL, TQ_ERR_SHAPE, TQ_ERR_EMPTY, TQ_ERR_CAPACITY = -1, -2, -3, -4
TQ_ERR_WORKSPACE, TQ_ERR_UNSUPPORTED, TQ_ERR_HIP, TQ_ERR_ALIGN = -5, -6, -7, -8


class TqKvCacheStruct(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero")] + \
               [(n, ctypes.c_int32) for n in ("batch", "n_kv_heads", "head_dim", "group_size", "capacity", "layout")]


class TqDecodeOptsStruct(ctypes.Structure):
    _fields_ = [("n_splits", ctypes.c_int32), ("variant", ctypes.c_int32), ("window", ctypes.c_int32),
                ("n_queries", ctypes.c_int32)]


class TqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tq_status_string(status)} (status {status})")


_lib = None


def library_path() -> Path:
    return _LIB_PATH


def raw():
    """The loaded ctypes library with argtypes set (tests use it to pass deliberately bad arguments)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise RuntimeError(f"{_LIB_PATH} is missing: the HIP library is not built "
                               "(run `python -m paper_2604_16957_amd.build`); there is no fallback path")
        L = ctypes.CDLL(str(_LIB_PATH))
        P, I, F, SZ = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        CP = ctypes.POINTER(TqKvCacheStruct)
        OP = ctypes.POINTER(TqDecodeOptsStruct)
        L.tq_quantize_kv.argtypes = [CP, P, P, I, I, P]
        L.tq_sdpa_int4_decode.argtypes = [CP, P, I, I, F, P, P, SZ, OP, P]
        L.tq_sdpa_int4_decode_static.argtypes = [CP, P, I, I, F, P, OP, P]
        L.tq_sdpa_int4_decode_static.restype = ctypes.c_int
        L.tq_quantize_kv_paged.argtypes = [CP, P, I, I, P, P, P, I, P]
        L.tq_sdpa_int4_decode_paged.argtypes = [CP, P, I, I, P, I, P, I, F, P, P, SZ, OP, P]
        L.tq_sdpa_int4_append_decode.argtypes = [CP, P, P, P, I, I, F, P, P, SZ, OP, P]
        L.tq_sdpa_int4_decode_varlen.argtypes = [CP, P, I, P, I, F, P, P, SZ, OP, P]
        L.tq_sdpa_int4_append_decode_varlen.argtypes = [CP, P, P, P, I, P, I, F, P, P, SZ, OP, P]
        L.tq_sdpa_int4_append_decode_paged.argtypes = [CP, P, I, I, P, P, P, I, P, I, F, P, P, SZ, OP, P]
        L.tq_quantize_kv_varlen.argtypes = [CP, P, P, P, I, P]
        L.tq_sdpa_int4_partial.argtypes = [CP, P, I, I, F, P, SZ, OP, ctypes.POINTER(ctypes.c_int32), P]
        L.tq_sdpa_int4_reduce.argtypes = [I, I, I, I, P, SZ, P, P]
        L.tq_dequant_then_attend.argtypes = [CP, P, I, I, F, P, P, SZ, P, SZ, OP, P]
        for f in (L.tq_quantize_kv, L.tq_sdpa_int4_decode, L.tq_sdpa_int4_partial, L.tq_sdpa_int4_reduce,
                  L.tq_dequant_then_attend):
            f.restype = ctypes.c_int
        L.tq_workspace_bytes.argtypes = [I, I, I]
        L.tq_workspace_bytes.restype = SZ
        L.tq_dense_scratch_bytes.argtypes = [I, I, I, I]
        L.tq_dense_scratch_bytes.restype = SZ
        L.tq_kv_bytes.argtypes = [I, I, I, I]
        L.tq_kv_bytes.restype = SZ
        L.tq_kv_bytes_grouped.argtypes = [I, I, I, I, I]
        L.tq_kv_bytes_grouped.restype = SZ
        L.tq_plan_splits.argtypes = [I, I, I]
        L.tq_plan_splits.restype = I
        L.tq_decode_launches.argtypes = [CP, I, I, F, OP]
        L.tq_decode_launches.restype = I
        L.tq_status_string.argtypes = [ctypes.c_int]
        L.tq_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def tq_status_string(status: int) -> str:
    return raw().tq_status_string(int(status)).decode()


def tq_workspace_bytes(batch: int, n_q_heads: int, head_dim: int) -> int:
    return int(raw().tq_workspace_bytes(batch, n_q_heads, head_dim))


def tq_dense_scratch_bytes(batch: int, n_kv_heads: int, seq_len: int, head_dim: int) -> int:
    return int(raw().tq_dense_scratch_bytes(batch, n_kv_heads, seq_len, head_dim))


def tq_kv_bytes(batch: int, n_kv_heads: int, capacity: int, head_dim: int) -> int:
    return int(raw().tq_kv_bytes(batch, n_kv_heads, capacity, head_dim))


def tq_kv_bytes_grouped(batch: int, n_kv_heads: int, capacity: int, head_dim: int, group_size: int) -> int:
    return int(raw().tq_kv_bytes_grouped(batch, n_kv_heads, capacity, head_dim, group_size))


def tq_plan_splits(batch: int, n_kv_heads: int, seq_len: int) -> int:
    return int(raw().tq_plan_splits(batch, n_kv_heads, seq_len))


def tq_decode_launches(cache: "KVCache", n_q_heads: int, seq_len: int, attn_scale: float, n_splits: int = 0,
                       variant: int = 0, window: int = 0, n_queries: int = 1) -> int:
    """Kernel launches one tq_sdpa_int4_decode call makes for this configuration (1 or 2; 0 = invalid)."""
    return int(raw().tq_decode_launches(ctypes.byref(cache.struct), int(n_q_heads), int(seq_len), float(attn_scale),
                                        _opts(n_splits, variant, window, n_queries)))


class KVCache:
    """Caller-owned cache for one layer: six torch tensors in the canonical layout of tq.h."""

    def __init__(self, batch: int, n_kv_heads: int, head_dim: int, capacity: int, device="cuda", group_size: int = 32):
        ng = head_dim // group_size
        self.group_size = group_size
        shape = (batch, n_kv_heads, capacity)
        self.k_codes = torch.empty(shape + (head_dim // 2,), dtype=torch.uint8, device=device)
        self.v_codes = torch.empty_like(self.k_codes)
        self.k_scale = torch.empty(shape + (ng,), dtype=torch.float16, device=device)
        self.k_zero = torch.empty_like(self.k_scale)
        self.v_scale = torch.empty_like(self.k_scale)
        self.v_zero = torch.empty_like(self.k_scale)
        self.batch, self.n_kv_heads, self.head_dim, self.capacity = batch, n_kv_heads, head_dim, capacity
        self.struct = TqKvCacheStruct(
            self.k_codes.data_ptr(), self.v_codes.data_ptr(), self.k_scale.data_ptr(), self.k_zero.data_ptr(),
            self.v_scale.data_ptr(), self.v_zero.data_ptr(), batch, n_kv_heads, head_dim, group_size, capacity, 0)

    def tensors(self):
        return (self.k_codes, self.k_scale, self.k_zero, self.v_codes, self.v_scale, self.v_zero)

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in self.tensors())


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _opts(n_splits: int, variant: int, window: int = 0, n_queries: int = 1):
    if not n_splits and not variant and not window and n_queries <= 1:
        return None
    return ctypes.byref(TqDecodeOptsStruct(int(n_splits), int(variant), int(window), int(n_queries)))


def _queries(q: torch.Tensor):
    """q is [B, H_q, d] (one query token per sequence) or [B, n_queries, H_q, d] -> (n_queries, H_q)."""
    if q.dim() == 4:
        return int(q.shape[1]), int(q.shape[2])
    return 1, int(q.shape[1])


def _check(rc: int, where: str):
    if rc != TQ_OK:
        raise TqError(rc, where)


def _need(t: torch.Tensor, dtype, name: str):
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of {dtype}")


def tq_quantize_kv(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor, pos: int, stream=None) -> None:
    """k_new, v_new: fp16 [B, H_kv, n_new, d]; written at token positions pos .. pos+n_new-1."""
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    if k_new.shape != v_new.shape or k_new.dim() != 4 or \
            tuple(k_new.shape[:2]) != (cache.batch, cache.n_kv_heads) or k_new.shape[3] != cache.head_dim:
        raise ValueError("k_new/v_new must be [batch, n_kv_heads, n_new, head_dim]")
    rc = raw().tq_quantize_kv(ctypes.byref(cache.struct), k_new.data_ptr(), v_new.data_ptr(), int(pos),
                              int(k_new.shape[2]), _stream_ptr(stream))
    _check(rc, "tq_quantize_kv")


def _workspace_for(cache: KVCache, n_q_heads: int, workspace, n_queries: int = 1):
    need = tq_workspace_bytes(cache.batch * n_queries, n_q_heads, cache.head_dim)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=cache.k_codes.device)
    return workspace, workspace.numel() * workspace.element_size()


def tq_sdpa_int4_decode(cache: KVCache, q: torch.Tensor, seq_len: int, attn_scale: float, out=None,
                        workspace=None, n_splits: int = 0, variant: int = 0, stream=None, window: int = 0) -> torch.Tensor:
    """q: fp16 [B, H_q, d] -> out fp16 [B, H_q, d]; or q [B, n_queries, H_q, d] = the sequence's last
    n_queries tokens, causal among themselves -> out of the same shape."""
    _need(q, torch.float16, "q")
    if out is None:
        out = torch.empty_like(q)
    nq, hq = _queries(q)
    workspace, wbytes = _workspace_for(cache, hq, workspace, nq)
    rc = raw().tq_sdpa_int4_decode(ctypes.byref(cache.struct), q.data_ptr(), hq, int(seq_len),
                                   float(attn_scale), out.data_ptr(), workspace.data_ptr(), wbytes,
                                   _opts(n_splits, variant, window, nq), _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_decode")
    return out


TQ_STATIC_SCRATCH_BYTES = 20 << 20


def tq_sdpa_int4_decode_static(cache: KVCache, q: torch.Tensor, seq_len: int, attn_scale: float, out: torch.Tensor,
                               n_splits: int = 0, variant: int = 0, stream=None, window: int = 0) -> torch.Tensor:
    """tq_sdpa_int4_decode without a workspace (the library's own static device array takes its place) and
    without any allocation: `out` has to be passed in."""
    _need(q, torch.float16, "q")
    _need(out, torch.float16, "out")
    nq, hq = _queries(q)
    rc = raw().tq_sdpa_int4_decode_static(ctypes.byref(cache.struct), q.data_ptr(), hq, int(seq_len),
                                          float(attn_scale), out.data_ptr(), _opts(n_splits, variant, window, nq),
                                          _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_decode_static")
    return out


def tq_sdpa_int4_append_decode(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, seq_len: int,
                               attn_scale: float, out=None, workspace=None, n_splits: int = 0, variant: int = 0,
                               stream=None, window: int = 0) -> torch.Tensor:
    """One decode step: k_new, v_new fp16 [B, H_kv, n_queries, d] are written at the end of the seq_len tokens,
    then q ([B, H_q, d], or [B, n_queries, H_q, d]) attends them."""
    _need(q, torch.float16, "q")
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    nq, hq = _queries(q)
    if k_new.shape != v_new.shape or tuple(k_new.shape) != (cache.batch, cache.n_kv_heads, nq, cache.head_dim):
        raise ValueError("k_new/v_new must be [batch, n_kv_heads, n_queries, head_dim]")
    if out is None:
        out = torch.empty_like(q)
    workspace, wbytes = _workspace_for(cache, hq, workspace, nq)
    rc = raw().tq_sdpa_int4_append_decode(ctypes.byref(cache.struct), k_new.data_ptr(), v_new.data_ptr(), q.data_ptr(),
                                          hq, int(seq_len), float(attn_scale), out.data_ptr(),
                                          workspace.data_ptr(), wbytes, _opts(n_splits, variant, window, nq),
                                          _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_append_decode")
    return out


def tq_sdpa_int4_decode_varlen(cache: KVCache, q: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                               attn_scale: float, out=None, workspace=None, n_splits: int = 0, variant: int = 0,
                               stream=None, window: int = 0) -> torch.Tensor:
    """q: fp16 [B, H_q, d] or [B, n_queries, H_q, d]; seq_lens: int32 device tensor [B] -> out like q."""
    _need(q, torch.float16, "q")
    _need(seq_lens, torch.int32, "seq_lens")
    if out is None:
        out = torch.empty_like(q)
    nq, hq = _queries(q)
    workspace, wbytes = _workspace_for(cache, hq, workspace, nq)
    rc = raw().tq_sdpa_int4_decode_varlen(ctypes.byref(cache.struct), q.data_ptr(), hq,
                                          seq_lens.data_ptr(), int(max_seq_len), float(attn_scale), out.data_ptr(),
                                          workspace.data_ptr(), wbytes, _opts(n_splits, variant, window, nq),
                                          _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_decode_varlen")
    return out


def tq_sdpa_int4_append_decode_varlen(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor,
                                      seq_lens: torch.Tensor, max_seq_len: int, attn_scale: float, out=None,
                                      workspace=None, n_splits: int = 0, variant: int = 0, stream=None,
                                      window: int = 0) -> torch.Tensor:
    """One decode step with per-sequence lengths (int32 device tensor [B], each counting the new token): k_new,
    v_new fp16 [B, H_kv, n_queries, d] go to the end of every sequence, then q attends."""
    _need(q, torch.float16, "q")
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    _need(seq_lens, torch.int32, "seq_lens")
    nq, hq = _queries(q)
    if k_new.shape != v_new.shape or tuple(k_new.shape) != (cache.batch, cache.n_kv_heads, nq, cache.head_dim):
        raise ValueError("k_new/v_new must be [batch, n_kv_heads, n_queries, head_dim]")
    if out is None:
        out = torch.empty_like(q)
    workspace, wbytes = _workspace_for(cache, hq, workspace, nq)
    rc = raw().tq_sdpa_int4_append_decode_varlen(ctypes.byref(cache.struct), k_new.data_ptr(), v_new.data_ptr(),
                                                 q.data_ptr(), hq, seq_lens.data_ptr(), int(max_seq_len),
                                                 float(attn_scale), out.data_ptr(), workspace.data_ptr(), wbytes,
                                                 _opts(n_splits, variant, window, nq), _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_append_decode_varlen")
    return out


def tq_sdpa_int4_append_decode_paged(pool: KVCache, block_table: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                                     q: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int, attn_scale: float,
                                     out=None, workspace=None, n_splits: int = 0, variant: int = 0, stream=None,
                                     window: int = 0) -> torch.Tensor:
    """The same over a pool of pages: block_table int32 [B, max_blocks] on the device."""
    _need(q, torch.float16, "q")
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    _need(seq_lens, torch.int32, "seq_lens")
    _need(block_table, torch.int32, "block_table")
    nq, hq = _queries(q)
    if out is None:
        out = torch.empty_like(q)
    need = tq_workspace_bytes(int(q.shape[0]) * nq, hq, pool.head_dim)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = raw().tq_sdpa_int4_append_decode_paged(ctypes.byref(pool.struct), block_table.data_ptr(),
                                                int(block_table.shape[1]), int(q.shape[0]), k_new.data_ptr(),
                                                v_new.data_ptr(), q.data_ptr(), hq, seq_lens.data_ptr(),
                                                int(max_seq_len), float(attn_scale), out.data_ptr(),
                                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                _opts(n_splits, variant, window, nq), _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_append_decode_paged")
    return out


def tq_quantize_kv_varlen(cache: KVCache, k_new: torch.Tensor, v_new: torch.Tensor, positions: torch.Tensor,
                          stream=None) -> None:
    """k_new, v_new: fp16 [B, H_kv, n_new, d]; positions: int32 device tensor [B]."""
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    _need(positions, torch.int32, "positions")
    rc = raw().tq_quantize_kv_varlen(ctypes.byref(cache.struct), k_new.data_ptr(), v_new.data_ptr(),
                                     positions.data_ptr(), int(k_new.shape[2]), _stream_ptr(stream))
    _check(rc, "tq_quantize_kv_varlen")


def tq_quantize_kv_paged(pool: KVCache, block_table: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                         positions: torch.Tensor, stream=None) -> None:
    """pool: a KVCache whose batch dimension counts pages; block_table int32 [B, max_blocks] (device);
    k_new, v_new fp16 [B, H_kv, n_new, d]; positions int32 [B] (device)."""
    _need(k_new, torch.float16, "k_new")
    _need(v_new, torch.float16, "v_new")
    _need(positions, torch.int32, "positions")
    _need(block_table, torch.int32, "block_table")
    rc = raw().tq_quantize_kv_paged(ctypes.byref(pool.struct), block_table.data_ptr(), int(block_table.shape[1]),
                                    int(block_table.shape[0]), k_new.data_ptr(), v_new.data_ptr(),
                                    positions.data_ptr(), int(k_new.shape[2]), _stream_ptr(stream))
    _check(rc, "tq_quantize_kv_paged")


def tq_sdpa_int4_decode_paged(pool: KVCache, block_table: torch.Tensor, q: torch.Tensor, seq_lens: torch.Tensor,
                              max_seq_len: int, attn_scale: float, out=None, workspace=None, n_splits: int = 0,
                              variant: int = 0, stream=None, window: int = 0) -> torch.Tensor:
    """q: fp16 [B, H_q, d] or [B, n_queries, H_q, d]; block_table int32 [B, max_blocks] and seq_lens int32 [B]
    on the device."""
    _need(q, torch.float16, "q")
    _need(seq_lens, torch.int32, "seq_lens")
    _need(block_table, torch.int32, "block_table")
    if out is None:
        out = torch.empty_like(q)
    nq, hq = _queries(q)
    need = tq_workspace_bytes(int(q.shape[0]) * nq, hq, pool.head_dim)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = raw().tq_sdpa_int4_decode_paged(ctypes.byref(pool.struct), block_table.data_ptr(), int(block_table.shape[1]),
                                         int(q.shape[0]), q.data_ptr(), hq, seq_lens.data_ptr(),
                                         int(max_seq_len), float(attn_scale), out.data_ptr(), workspace.data_ptr(),
                                         workspace.numel() * workspace.element_size(), _opts(n_splits, variant, window, nq),
                                         _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_decode_paged")
    return out


def tq_sdpa_int4_partial(cache: KVCache, q: torch.Tensor, seq_len: int, attn_scale: float, workspace: torch.Tensor,
                         n_splits: int = 0, variant: int = 0, stream=None, window: int = 0) -> int:
    """Phase 1 only; returns the number of chunks written into workspace."""
    _need(q, torch.float16, "q")
    n = ctypes.c_int32(0)
    nq, hq = _queries(q)
    rc = raw().tq_sdpa_int4_partial(ctypes.byref(cache.struct), q.data_ptr(), hq, int(seq_len),
                                    float(attn_scale), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _opts(n_splits, variant, window, nq),
                                    ctypes.byref(n), _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_partial")
    return n.value


def tq_sdpa_int4_reduce(batch: int, n_q_heads: int, head_dim: int, n_splits: int, workspace: torch.Tensor,
                        out: torch.Tensor, stream=None) -> torch.Tensor:
    rc = raw().tq_sdpa_int4_reduce(batch, n_q_heads, head_dim, n_splits, workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), out.data_ptr(), _stream_ptr(stream))
    _check(rc, "tq_sdpa_int4_reduce")
    return out


def tq_dequant_then_attend(cache: KVCache, q: torch.Tensor, seq_len: int, attn_scale: float, out=None,
                           workspace=None, dense_scratch=None, n_splits: int = 0, stream=None,
                           variant: int = 0) -> torch.Tensor:
    """The unfused comparator; variant 1 = its attention phase on the generic vector-ALU kernel."""
    _need(q, torch.float16, "q")
    if out is None:
        out = torch.empty_like(q)
    workspace, wbytes = _workspace_for(cache, q.shape[1], workspace)
    if dense_scratch is None:
        dense_scratch = torch.empty(tq_dense_scratch_bytes(cache.batch, cache.n_kv_heads, seq_len, cache.head_dim),
                                    dtype=torch.uint8, device=q.device)
    rc = raw().tq_dequant_then_attend(ctypes.byref(cache.struct), q.data_ptr(), int(q.shape[1]), int(seq_len),
                                      float(attn_scale), out.data_ptr(), workspace.data_ptr(), wbytes,
                                      dense_scratch.data_ptr(), dense_scratch.numel() * dense_scratch.element_size(),
                                      _opts(n_splits, variant), _stream_ptr(stream))
    _check(rc, "tq_dequant_then_attend")
    return out
