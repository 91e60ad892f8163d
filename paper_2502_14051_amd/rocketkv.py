"""Thin ctypes binding of ``librocketkv.so`` (see ``include/rocketkv.h``).

Argument marshalling only: every function here forwards device pointers of
torch tensors to the C ABI entry point of the same name and raises
``RocketKVError`` on a non-zero status.  torch is used for device memory and
for the current HIP stream; no computation of the method happens in Python and
there is no fallback: if the native library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librocketkv.so")

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR = 0, -1, -2, -3, -4
OP_HSA_DECODE, OP_DENSE_DECODE, OP_SNAPKV, OP_ATTEND = 0, 1, 2, 3
MAX_PAGES = 32768
V_CHANNEL_MAJOR, V_TOKEN_MAJOR = 0, 1

EXPORTS = [
    "rocketkv_workspace_bytes", "rocketkv_workspace_init", "rocketkv_build_page_summaries", "rocketkv_hsa_select",
    "rocketkv_attend", "rocketkv_hsa_decode", "rocketkv_hsa_decode_append", "rocketkv_dense_decode", "rocketkv_append_kv",
    "rocketkv_snapkv_compress", "rocketkv_decompose", "rocketkv_last_error", "rocketkv_version",
    "rocketkv_snapkv_filter", "rocketkv_mt_build_page_summaries", "rocketkv_mt_workspace_bytes", "rocketkv_mt_hsa_decode",
    "rocketkv_mt_append_kv", "rocketkv_mt_hsa_decode_append",
    "rocketkv_stream_read", "rocketkv_stream_read_sink_bytes", "rocketkv_hsa_decode_noalloc",
    "rocketkv_stream_gather", "rocketkv_stream_gather_sink_bytes",
]
NOALLOC_SCRATCH_BYTES = 4 << 20


class RocketKVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rocketkv status {status}: {message}")
        self.status = status


class CacheStruct(C.Structure):
    """Mirror of ``rocketkv_cache_t``."""
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("page_size", C.c_int32), ("pages_cap", C.c_int32),
        ("n_phys_pages", C.c_int64), ("stride_page", C.c_int64), ("stride_head", C.c_int64),
        ("seq_lens", C.c_void_p), ("block_table", C.c_void_p),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("v_layout", C.c_int32),
    ]


class IndexStruct(C.Structure):
    """Mirror of ``rocketkv_index_t``."""
    _fields_ = [("token_index", C.c_void_p), ("n_indexed", C.c_void_p), ("page_size", C.c_int32),
                ("pages_cap", C.c_int32)]


class SplitStruct(C.Structure):
    """Mirror of ``rocketkv_split_t``."""
    _fields_ = [
        ("c", C.c_double), ("r", C.c_double), ("stage1", C.c_double), ("stage2", C.c_double),
        ("head_ratio", C.c_double), ("page_size", C.c_int32), ("keep_budget", C.c_int32),
        ("channel_budget", C.c_int32), ("attend_tokens", C.c_int32),
        ("storage", C.c_double), ("storage_mt", C.c_double), ("traffic", C.c_double),
    ]


_lib = None


def lib():
    """Load the native library (built by ``paper_2502_14051_amd.build``)."""
    global _lib
    if _lib is None:
        # torch first: the library must bind to the HIP runtime torch has already loaded, so that
        # streams and device pointers are shared with it
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2502_14051_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        cp = C.POINTER(CacheStruct)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.rocketkv_workspace_bytes.restype = sz
        L.rocketkv_workspace_bytes.argtypes = [i32, cp, i32, i32]
        L.rocketkv_workspace_init.restype = i32
        L.rocketkv_workspace_init.argtypes = [vp, sz, vp]
        L.rocketkv_build_page_summaries.restype = i32
        L.rocketkv_build_page_summaries.argtypes = [cp, vp, vp, i32, i32, vp]
        L.rocketkv_hsa_select.restype = i32
        L.rocketkv_hsa_select.argtypes = [cp, vp, vp, vp, i32, i32, i32, vp, i32, vp, vp, vp]
        L.rocketkv_attend.restype = i32
        L.rocketkv_attend.argtypes = [cp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.rocketkv_hsa_decode.restype = i32
        L.rocketkv_hsa_decode.argtypes = [cp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.rocketkv_stream_gather.restype = i32
        L.rocketkv_stream_gather.argtypes = [cp, vp, i32, vp, vp]
        L.rocketkv_stream_gather_sink_bytes.restype = sz
        L.rocketkv_stream_gather_sink_bytes.argtypes = [cp, i32]
        L.rocketkv_hsa_decode_noalloc.restype = i32
        L.rocketkv_hsa_decode_noalloc.argtypes = [cp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.rocketkv_hsa_decode_append.restype = i32
        L.rocketkv_hsa_decode_append.argtypes = [cp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.rocketkv_dense_decode.restype = i32
        L.rocketkv_dense_decode.argtypes = [cp, vp, vp, vp, vp, sz, vp]
        L.rocketkv_append_kv.restype = i32
        L.rocketkv_append_kv.argtypes = [cp, vp, vp, vp, vp, vp]
        L.rocketkv_snapkv_compress.restype = i32
        L.rocketkv_snapkv_compress.argtypes = [vp, cp, i32, i32, i32, cp, vp, vp, sz, vp]
        ip = C.POINTER(IndexStruct)
        L.rocketkv_snapkv_filter.restype = i32
        L.rocketkv_snapkv_filter.argtypes = [vp, cp, i32, i32, i32, ip, vp, sz, vp]
        L.rocketkv_mt_build_page_summaries.restype = i32
        L.rocketkv_mt_build_page_summaries.argtypes = [cp, ip, vp, vp, i32, i32, vp]
        L.rocketkv_mt_workspace_bytes.restype = sz
        L.rocketkv_mt_workspace_bytes.argtypes = [cp, ip, i32]
        L.rocketkv_mt_hsa_decode.restype = i32
        L.rocketkv_mt_hsa_decode.argtypes = [cp, ip, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.rocketkv_mt_append_kv.restype = i32
        L.rocketkv_mt_append_kv.argtypes = [cp, ip, vp, vp, vp, vp, vp]
        L.rocketkv_mt_hsa_decode_append.restype = i32
        L.rocketkv_mt_hsa_decode_append.argtypes = [cp, ip, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.rocketkv_decompose.restype = i32
        L.rocketkv_decompose.argtypes = [C.c_int64, i32, i32, C.POINTER(SplitStruct)]
        L.rocketkv_last_error.restype = C.c_char_p
        L.rocketkv_last_error.argtypes = []
        L.rocketkv_version.restype = i32
        L.rocketkv_version.argtypes = []
        L.rocketkv_stream_read.restype = i32
        L.rocketkv_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.rocketkv_stream_read_sink_bytes.restype = C.c_size_t
        L.rocketkv_stream_read_sink_bytes.argtypes = []
        _lib = L
    return _lib


def last_error() -> str:
    return lib().rocketkv_last_error().decode()


def _check(status: int):
    if status != OK:
        raise RocketKVError(status, last_error())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


@dataclass
class Cache:
    """A paged KV cache living in torch tensors, plus its C descriptor.

    k_pool: bf16 [n_phys_pages][n_kv_heads][page_size][head_dim]
    v_pool: bf16 [n_phys_pages][n_kv_heads][head_dim][page_size], or
            [n_phys_pages][n_kv_heads][page_size][head_dim] when v_layout is V_TOKEN_MAJOR
    Both may be strided views of one allocation (`interleaved`: the K tile of a (page, head) is
    followed by its V tile), which the C descriptor expresses through its strides.
    seq_lens: int32 [batch]; block_table: int32 [batch][pages_cap] or None (identity).
    """
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_size: int
    pages_cap: int
    k_pool: object
    v_pool: object
    seq_lens: object
    block_table: object = None
    v_layout: int = V_CHANNEL_MAJOR

    def struct(self) -> CacheStruct:
        assert self.k_pool.stride()[:2] == self.v_pool.stride()[:2], "K and V pools must share strides"
        return CacheStruct(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim,
                           self.page_size, self.pages_cap, int(self.k_pool.shape[0]),
                           int(self.k_pool.stride(0)), int(self.k_pool.stride(1)), _ptr(self.seq_lens),
                           _ptr(self.block_table), _ptr(self.k_pool), _ptr(self.v_pool), self.v_layout)

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads


def alloc_cache(batch, n_q_heads, n_kv_heads, head_dim, page_size, pages_cap, device,
                block_table=None, n_phys_pages=None, zero=False, v_layout=V_CHANNEL_MAJOR,
                interleaved=False) -> Cache:
    import torch
    pages_cap = (pages_cap + 7) // 8 * 8
    n_phys = n_phys_pages if n_phys_pages is not None else batch * pages_cap
    mk = torch.zeros if zero else torch.empty
    v_shape = (page_size, head_dim) if v_layout == V_TOKEN_MAJOR else (head_dim, page_size)
    if interleaved:
        both = mk((n_phys, n_kv_heads, 2, page_size * head_dim), dtype=torch.bfloat16, device=device)
        k_pool = both[:, :, 0].view(n_phys, n_kv_heads, page_size, head_dim)
        v_pool = both[:, :, 1].view((n_phys, n_kv_heads) + v_shape)
    else:
        k_pool = mk((n_phys, n_kv_heads, page_size, head_dim), dtype=torch.bfloat16, device=device)
        v_pool = mk((n_phys, n_kv_heads) + v_shape, dtype=torch.bfloat16, device=device)
    seq_lens = torch.zeros((batch,), dtype=torch.int32, device=device)
    return Cache(batch, n_q_heads, n_kv_heads, head_dim, page_size, pages_cap, k_pool, v_pool,
                 seq_lens, block_table, v_layout)


def pack_cache(K, V, seq_lens, n_q_heads, page_size, pages_cap=None, block_table=None,
               n_phys_pages=None, v_layout=V_CHANNEL_MAJOR, interleaved=False) -> Cache:
    """Lay token-major bf16 K, V ([B][Hkv][n][D] torch tensors on the device) out as a paged cache.

    Pure data movement (pad, reshape, permute, scatter by the block table)."""
    import torch
    B, Hkv, n, D = K.shape
    need = (n + page_size - 1) // page_size
    pages_cap = max(need, pages_cap or 0, 1)
    cache = alloc_cache(B, n_q_heads, Hkv, D, page_size, pages_cap, K.device, block_table,
                        n_phys_pages, zero=True, v_layout=v_layout, interleaved=interleaved)
    pc = cache.pages_cap
    pad = pc * page_size - n
    Kp = torch.nn.functional.pad(K, (0, 0, 0, pad)) if pad else K
    Vp = torch.nn.functional.pad(V, (0, 0, 0, pad)) if pad else V
    Kt = Kp.reshape(B, Hkv, pc, page_size, D).permute(0, 2, 1, 3, 4)        # [B][pc][Hkv][ps][D]
    Vt = Vp.reshape(B, Hkv, pc, page_size, D).permute(0, 2, 1, 3, 4)        # [B][pc][Hkv][ps][D]
    if v_layout != V_TOKEN_MAJOR:
        Vt = Vt.transpose(3, 4)                                              # [B][pc][Hkv][D][ps]
    v_tile = tuple(cache.v_pool.shape[2:])
    if block_table is None:
        cache.k_pool[:B * pc].copy_(Kt.reshape(B * pc, Hkv, page_size, D))
        cache.v_pool[:B * pc].copy_(Vt.reshape((B * pc, Hkv) + v_tile))
    else:
        idx = block_table.reshape(-1).long()
        cache.k_pool.index_copy_(0, idx, Kt.reshape(B * pc, Hkv, page_size, D).contiguous())
        cache.v_pool.index_copy_(0, idx, Vt.reshape((B * pc, Hkv) + v_tile).contiguous())
    cache.seq_lens.copy_(torch.as_tensor(seq_lens, dtype=torch.int32))
    return cache


def unpack_cache(cache: Cache):
    """Inverse of pack_cache: token-major K, V [B][Hkv][pages_cap*page_size][D] (data movement)."""
    B, Hkv, ps, D, pc = cache.batch, cache.n_kv_heads, cache.page_size, cache.head_dim, cache.pages_cap
    if cache.block_table is None:
        kp, vp = cache.k_pool[:B * pc], cache.v_pool[:B * pc]
    else:
        idx = cache.block_table.reshape(-1).long()
        kp, vp = cache.k_pool[idx], cache.v_pool[idx]
    K = kp.reshape(B, pc, Hkv, ps, D).permute(0, 2, 1, 3, 4).reshape(B, Hkv, pc * ps, D)
    if cache.v_layout == V_TOKEN_MAJOR:
        V = vp.reshape(B, pc, Hkv, ps, D).permute(0, 2, 1, 3, 4).reshape(B, Hkv, pc * ps, D)
    else:
        V = vp.reshape(B, pc, Hkv, D, ps).permute(0, 2, 1, 4, 3).reshape(B, Hkv, pc * ps, D)
    return K.contiguous(), V.contiguous()


def alloc_summaries(cache: Cache):
    import torch
    shape = (cache.batch, cache.n_kv_heads, cache.head_dim, cache.pages_cap)
    return (torch.zeros(shape, dtype=torch.bfloat16, device=cache.k_pool.device),
            torch.zeros(shape, dtype=torch.bfloat16, device=cache.k_pool.device))


def workspace_bytes(op: int, cache: Cache, a: int = 0, b: int = 0) -> int:
    st = cache.struct()
    n = lib().rocketkv_workspace_bytes(op, C.byref(st), a, b)
    if n == 0 and last_error():
        raise RocketKVError(INVALID_ARG, last_error())
    return int(n)


def workspace_init(workspace, stream=None):
    _check(lib().rocketkv_workspace_init(_ptr(workspace), workspace.numel(), _stream(stream)))


def alloc_workspace(op: int, cache: Cache, a: int = 0, b: int = 0, stream=None):
    """Allocate (torch) and initialise a workspace for `op` on `cache`."""
    import torch
    n = workspace_bytes(op, cache, a, b)
    ws = torch.empty((max(n, 256),), dtype=torch.uint8, device=cache.k_pool.device)
    workspace_init(ws, stream)
    return ws


def build_page_summaries(cache: Cache, kmax, kmin, first_page: int = 0, n_pages: int = -1,
                         stream=None):
    st = cache.struct()
    _check(lib().rocketkv_build_page_summaries(C.byref(st), _ptr(kmax), _ptr(kmin), first_page,
                                               n_pages, _stream(stream)))


def hsa_select(cache: Cache, q, kmax, kmin, channel_budget: int, token_budget: int,
               n_recent_pages: int, out_pages, out_channels=None, out_scores=None, stream=None):
    st = cache.struct()
    _check(lib().rocketkv_hsa_select(C.byref(st), _ptr(q), _ptr(kmax), _ptr(kmin), channel_budget,
                                     token_budget, n_recent_pages, _ptr(out_pages),
                                     int(out_pages.shape[-1]), _ptr(out_channels),
                                     _ptr(out_scores), _stream(stream)))


def attend(cache: Cache, q, pages, out, out_lse, workspace, stream=None):
    st = cache.struct()
    row_len = 0 if pages is None else int(pages.shape[-1])
    _check(lib().rocketkv_attend(C.byref(st), _ptr(q), _ptr(pages), row_len, _ptr(out),
                                 _ptr(out_lse), _ptr(workspace), workspace.numel(),
                                 _stream(stream)))


def hsa_decode(cache: Cache, q, kmax, kmin, channel_budget: int, token_budget: int,
               n_recent_pages: int, out, out_lse, out_pages, out_channels, workspace, stream=None):
    st = cache.struct()
    _check(lib().rocketkv_hsa_decode(C.byref(st), _ptr(q), _ptr(kmax), _ptr(kmin), channel_budget,
                                     token_budget, n_recent_pages, _ptr(out), _ptr(out_lse),
                                     _ptr(out_pages), _ptr(out_channels), _ptr(workspace),
                                     workspace.numel(), _stream(stream)))


def hsa_decode_noalloc(cache: Cache, q, kmax, kmin, channel_budget: int, token_budget: int,
                       n_recent_pages: int, out, out_lse, out_pages, out_channels, stream=None):
    """rocketkv_hsa_decode on the library's own scratch buffer (no workspace, no allocation)."""
    st = cache.struct()
    _check(lib().rocketkv_hsa_decode_noalloc(C.byref(st), _ptr(q), _ptr(kmax), _ptr(kmin), channel_budget,
                                             token_budget, n_recent_pages, _ptr(out), _ptr(out_lse),
                                             _ptr(out_pages), _ptr(out_channels), _stream(stream)))


def hsa_decode_append(cache: Cache, q, k_new, v_new, kmax, kmin, channel_budget: int, token_budget: int,
                      n_recent_pages: int, out, out_lse, out_pages, out_channels, workspace, stream=None):
    st = cache.struct()
    _check(lib().rocketkv_hsa_decode_append(C.byref(st), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kmax),
                                            _ptr(kmin), channel_budget, token_budget, n_recent_pages,
                                            _ptr(out), _ptr(out_lse), _ptr(out_pages), _ptr(out_channels),
                                            _ptr(workspace), workspace.numel(), _stream(stream)))


def dense_decode(cache: Cache, q, out, out_lse, workspace, stream=None):
    st = cache.struct()
    _check(lib().rocketkv_dense_decode(C.byref(st), _ptr(q), _ptr(out), _ptr(out_lse),
                                       _ptr(workspace), workspace.numel(), _stream(stream)))


def append_kv(cache: Cache, k_new, v_new, kmax, kmin, stream=None):
    st = cache.struct()
    _check(lib().rocketkv_append_kv(C.byref(st), _ptr(k_new), _ptr(v_new), _ptr(kmax), _ptr(kmin),
                                    _stream(stream)))


def snapkv_compress(q_obs, src: Cache, window: int, pool_kernel: int, keep_budget: int,
                    dst: Cache, kept_idx, workspace, stream=None):
    s, d = src.struct(), dst.struct()
    _check(lib().rocketkv_snapkv_compress(_ptr(q_obs), C.byref(s), window, pool_kernel, keep_budget,
                                          C.byref(d), _ptr(kept_idx), _ptr(workspace),
                                          workspace.numel(), _stream(stream)))


@dataclass
class Index:
    """The logical sequence of RocketKV-MT in torch tensors, plus its C descriptor.

    token_index: int32 [batch][n_kv_heads][pages_cap * page_size]; n_indexed: int32 [batch]."""
    token_index: object
    n_indexed: object
    page_size: int
    pages_cap: int

    def struct(self) -> IndexStruct:
        return IndexStruct(_ptr(self.token_index), _ptr(self.n_indexed), self.page_size, self.pages_cap)


def alloc_index(cache: Cache, page_size: int, capacity_tokens: int) -> Index:
    import torch
    pages_cap = ((capacity_tokens + page_size - 1) // page_size + 7) // 8 * 8
    dev = cache.k_pool.device
    return Index(torch.full((cache.batch, cache.n_kv_heads, pages_cap * page_size), -1, dtype=torch.int32, device=dev),
                 torch.zeros((cache.batch,), dtype=torch.int32, device=dev), page_size, pages_cap)


def alloc_index_summaries(cache: Cache, index: Index):
    import torch
    shape = (cache.batch, cache.n_kv_heads, cache.head_dim, index.pages_cap)
    return (torch.zeros(shape, dtype=torch.bfloat16, device=cache.k_pool.device),
            torch.zeros(shape, dtype=torch.bfloat16, device=cache.k_pool.device))


def snapkv_filter(q_obs, src: Cache, window: int, pool_kernel: int, keep_budget: int, index: Index,
                  workspace, stream=None):
    st, ix = src.struct(), index.struct()
    _check(lib().rocketkv_snapkv_filter(_ptr(q_obs), C.byref(st), window, pool_kernel, keep_budget, C.byref(ix),
                                        _ptr(workspace), workspace.numel(), _stream(stream)))


def mt_build_page_summaries(cache: Cache, index: Index, kmax, kmin, first_page: int = 0, n_pages: int = -1,
                            stream=None):
    st, ix = cache.struct(), index.struct()
    _check(lib().rocketkv_mt_build_page_summaries(C.byref(st), C.byref(ix), _ptr(kmax), _ptr(kmin), first_page,
                                                  n_pages, _stream(stream)))


def mt_alloc_workspace(cache: Cache, index: Index, token_budget: int, stream=None):
    import torch
    st, ix = cache.struct(), index.struct()
    n = lib().rocketkv_mt_workspace_bytes(C.byref(st), C.byref(ix), token_budget)
    if n == 0:
        raise RocketKVError(INVALID_ARG, last_error())
    ws = torch.empty((max(int(n), 256),), dtype=torch.uint8, device=cache.k_pool.device)
    workspace_init(ws, stream)
    return ws


def mt_hsa_decode(cache: Cache, index: Index, q, kmax, kmin, channel_budget: int, token_budget: int,
                  n_recent_pages: int, out, out_lse, out_pages, out_channels, workspace, stream=None):
    st, ix = cache.struct(), index.struct()
    _check(lib().rocketkv_mt_hsa_decode(C.byref(st), C.byref(ix), _ptr(q), _ptr(kmax), _ptr(kmin), channel_budget,
                                        token_budget, n_recent_pages, _ptr(out), _ptr(out_lse), _ptr(out_pages),
                                        _ptr(out_channels), _ptr(workspace), workspace.numel(), _stream(stream)))


def mt_append_kv(cache: Cache, index: Index, k_new, v_new, kmax, kmin, stream=None):
    st, ix = cache.struct(), index.struct()
    _check(lib().rocketkv_mt_append_kv(C.byref(st), C.byref(ix), _ptr(k_new), _ptr(v_new), _ptr(kmax), _ptr(kmin),
                                       _stream(stream)))


def mt_hsa_decode_append(cache: Cache, index: Index, q, k_new, v_new, kmax, kmin, channel_budget: int,
                         token_budget: int, n_recent_pages: int, out, out_lse, out_pages, out_channels,
                         workspace, stream=None):
    st, ix = cache.struct(), index.struct()
    _check(lib().rocketkv_mt_hsa_decode_append(C.byref(st), C.byref(ix), _ptr(q), _ptr(k_new), _ptr(v_new),
                                               _ptr(kmax), _ptr(kmin), channel_budget, token_budget,
                                               n_recent_pages, _ptr(out), _ptr(out_lse), _ptr(out_pages),
                                               _ptr(out_channels), _ptr(workspace), workspace.numel(),
                                               _stream(stream)))


def decompose(seq_len: int, token_budget: int, head_dim: int = 128) -> dict:
    """Adaptive compression decomposition (host arithmetic in the library); see rocketkv_decompose."""
    out = SplitStruct()
    _check(lib().rocketkv_decompose(int(seq_len), int(token_budget), int(head_dim), C.byref(out)))
    return {name: getattr(out, name) for name, _ in SplitStruct._fields_}


def pages_row_len(cache: Cache, token_budget: int) -> int:
    """Row length of the page list hsa_decode / hsa_select write for this budget."""
    return max(1, min(cache.pages_cap, (token_budget + cache.page_size - 1) // cache.page_size))


def stream_gather(cache: Cache, pages, sink=None, stream=None):
    """Measurement aid: the K/V tiles of a page list read the way the attention kernels read them, nothing
    computed (see rocketkv_stream_gather).  Returns the sink tensor."""
    import torch
    st = cache.struct()
    if sink is None:
        sink = torch.empty((lib().rocketkv_stream_gather_sink_bytes(C.byref(st), pages.shape[-1]),), dtype=torch.uint8,
                           device=pages.device)
    _check(lib().rocketkv_stream_gather(C.byref(st), _ptr(pages), pages.shape[-1], _ptr(sink), _stream(stream)))
    return sink


def stream_read(buf, sink=None, stream=None):
    """Measurement aid: one streaming read of the whole tensor ``buf`` (see rocketkv_stream_read)."""
    import torch

    nbytes = buf.numel() * buf.element_size()
    if sink is None:
        sink = torch.empty((lib().rocketkv_stream_read_sink_bytes(),), dtype=torch.uint8, device=buf.device)
    _check(lib().rocketkv_stream_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream)))
    return sink
