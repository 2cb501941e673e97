"""ctypes binding of libsamkv.so: the same five entry points as include/samkv.h, taking torch tensors.

Argument marshalling only: every step of the path runs in the HIP kernels of the library.  torch is
used for device memory and for the current stream.  If the library is missing the import of this
module fails; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch  # noqa: F401  (must be loaded first: the library binds to the HIP runtime torch ships)

SAMKV_F32, SAMKV_BF16 = 0, 1
SAMKV_MAX_CTX, SAMKV_MAX_LEN = 128, 65536
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libsamkv.so")

EXPORTS = ("samkv_strerror", "samkv_kept_count", "samkv_kept_count_mid", "samkv_top_p", "samkv_workspace_bytes",
           "samkv_score", "samkv_score_noalloc", "samkv_score_select", "samkv_score_select_gather", "samkv_topk_select", "samkv_topk_select_v", "samkv_gather_v",
           "samkv_gather_q_v", "samkv_block_scores", "samkv_block_workspace_bytes", "samkv_block_select",
           "samkv_block_select_filter", "samkv_block_filter_count", "samkv_block_select_count", "samkv_gather_g", "samkv_gather_q_g",
           "samkv_gather", "samkv_gather_q", "samkv_recompute_attn", "samkv_query_attn", "samkv_recompute_query_attn", "samkv_query_attn_self",
           "samkv_kv_update", "samkv_peak_mfma_bf16", "samkv_peak_mfma_bf16_data", "samkv_peak_copy", "samkv_peak_read")
SAMKV_OVERWRITE, SAMKV_FUSION = 0, 1


class _Caches(ctypes.Structure):
    _fields_ = [
        ("n_ctx", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("len", ctypes.POINTER(ctypes.c_int32)),
        ("k", ctypes.POINTER(ctypes.c_void_p)), ("v", ctypes.POINTER(ctypes.c_void_p)),
    ]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2508_11661_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    cp = ctypes.POINTER(_Caches)
    lib.samkv_strerror.restype = ctypes.c_char_p
    lib.samkv_strerror.argtypes = [ctypes.c_int]
    lib.samkv_kept_count.restype = i32
    lib.samkv_kept_count.argtypes = [i32, f32]
    lib.samkv_workspace_bytes.restype = sz
    lib.samkv_workspace_bytes.argtypes = [i32] * 6
    lib.samkv_score.restype = ctypes.c_int
    lib.samkv_score.argtypes = [cp, vp, i32, vp, i32, vp, vp, sz, vp]
    lib.samkv_score_noalloc.restype = ctypes.c_int
    lib.samkv_score_noalloc.argtypes = [cp, vp, i32, vp, i32, vp, vp]
    lib.samkv_score_select.restype = ctypes.c_int
    lib.samkv_score_select.argtypes = [cp, vp, i32, vp, i32, f32, i32, i32, vp, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.samkv_score_select_gather.restype = ctypes.c_int
    lib.samkv_score_select_gather.argtypes = [cp, vp, i32, vp, i32, f32, i32, i32, vp, vp, vp, ctypes.POINTER(i32), vp, vp,
                                              vp, sz, vp]
    lib.samkv_topk_select.restype = ctypes.c_int
    lib.samkv_topk_select.argtypes = [vp, cp, f32, i32, i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.samkv_gather.restype = ctypes.c_int
    lib.samkv_gather.argtypes = [cp, vp, f32, vp, vp, vp]
    lib.samkv_kept_count_mid.restype = i32
    lib.samkv_kept_count_mid.argtypes = [i32, f32, i32, i32]
    lib.samkv_top_p.restype = ctypes.c_int
    lib.samkv_top_p.argtypes = [ctypes.POINTER(f32)] * 3 + [i32, i32, ctypes.POINTER(f32)]
    lib.samkv_topk_select_v.restype = ctypes.c_int
    lib.samkv_topk_select_v.argtypes = [vp, cp, ctypes.POINTER(f32), i32, i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.samkv_gather_v.restype = ctypes.c_int
    lib.samkv_gather_v.argtypes = [cp, vp, ctypes.POINTER(i32), vp, vp, vp]
    lib.samkv_gather_q_v.restype = ctypes.c_int
    lib.samkv_gather_q_v.argtypes = [cp, ctypes.POINTER(ctypes.c_void_p), vp, ctypes.POINTER(i32), vp, vp]
    lib.samkv_block_scores.restype = ctypes.c_int
    lib.samkv_block_scores.argtypes = [vp, cp, i32, vp, vp]
    lib.samkv_block_workspace_bytes.restype = sz
    lib.samkv_block_workspace_bytes.argtypes = [cp, i32]
    lib.samkv_block_select.restype = ctypes.c_int
    lib.samkv_block_select.argtypes = [vp, cp, i32, ctypes.POINTER(f32), i32, i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.samkv_block_select_filter.restype = ctypes.c_int
    lib.samkv_block_select_filter.argtypes = [vp, cp, i32, ctypes.POINTER(f32), i32, i32, vp, vp, sz, vp]
    lib.samkv_block_select_count.restype = i32
    lib.samkv_block_select_count.argtypes = [cp, i32, ctypes.POINTER(f32), i32, i32]
    lib.samkv_block_filter_count.restype = i32
    lib.samkv_block_filter_count.argtypes = [cp, i32, ctypes.POINTER(f32), i32, i32]
    lib.samkv_gather_g.restype = ctypes.c_int
    lib.samkv_gather_g.argtypes = [cp, vp, i32, vp, vp, vp]
    lib.samkv_gather_q_g.restype = ctypes.c_int
    lib.samkv_gather_q_g.argtypes = [cp, ctypes.POINTER(ctypes.c_void_p), vp, i32, vp, vp]
    lib.samkv_gather_q.restype = ctypes.c_int
    lib.samkv_gather_q.argtypes = [cp, ctypes.POINTER(ctypes.c_void_p), vp, f32, vp, vp]
    lib.samkv_recompute_attn.restype = ctypes.c_int
    lib.samkv_recompute_attn.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.samkv_query_attn.restype = ctypes.c_int
    lib.samkv_query_attn.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.samkv_recompute_query_attn.restype = ctypes.c_int
    lib.samkv_recompute_query_attn.argtypes = [vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.samkv_query_attn_self.restype = ctypes.c_int
    lib.samkv_query_attn_self.argtypes = [vp, i32, vp, vp, i32, vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, sz, vp]
    lib.samkv_peak_mfma_bf16.restype = ctypes.c_int
    lib.samkv_peak_mfma_bf16.argtypes = [vp, i32, i32, vp]
    lib.samkv_peak_mfma_bf16_data.restype = ctypes.c_int
    lib.samkv_peak_mfma_bf16_data.argtypes = [vp, i32, i32, i32, vp]
    lib.samkv_peak_copy.restype = ctypes.c_int
    lib.samkv_peak_copy.argtypes = [vp, vp, sz, vp]
    lib.samkv_peak_read.restype = ctypes.c_int
    lib.samkv_peak_read.argtypes = [vp, sz, vp, vp]
    lib.samkv_kv_update.restype = ctypes.c_int
    lib.samkv_kv_update.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
    return lib


_lib = _load()


class SamKVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {_lib.samkv_strerror(code).decode()} ({code})")


def _check(code: int, where: str) -> None:
    if code != 0:
        raise SamKVError(code, where)


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return SAMKV_F32
    if t == torch.bfloat16:
        return SAMKV_BF16
    raise TypeError(f"unsupported dtype {t}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be dense"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def upload(a, dtype: str) -> torch.Tensor:
    """numpy float32 array whose values are exact in `dtype` ("f32" or "bf16") -> dense device tensor of that dtype."""
    t = torch.from_numpy(__import__("numpy").ascontiguousarray(a)).cuda()
    return t.to({"f32": torch.float32, "bf16": torch.bfloat16}[dtype]).contiguous()


@dataclass
class Caches:
    """The per-document K/V caches of one layer: k[i], v[i] are [Hkv, L_i, d] device tensors."""

    k: Sequence[torch.Tensor]
    v: Optional[Sequence[torch.Tensor]]
    n_q_heads: int

    def __post_init__(self):
        k0 = self.k[0]
        self.n_ctx = len(self.k)
        self.n_kv_heads, _, self.head_dim = k0.shape
        self.dtype = _dtype_code(k0.dtype)
        self.lens = [int(t.shape[1]) for t in self.k]
        for t in list(self.k) + list(self.v or []):
            assert t.is_cuda and t.is_contiguous() and t.dtype == k0.dtype
            assert t.shape[0] == self.n_kv_heads and t.shape[2] == self.head_dim
        self._len = (ctypes.c_int32 * self.n_ctx)(*self.lens)
        self._k = (ctypes.c_void_p * self.n_ctx)(*[t.data_ptr() for t in self.k])
        self._v = (ctypes.c_void_p * self.n_ctx)(*[t.data_ptr() for t in self.v]) if self.v is not None else None
        self.c = _Caches(self.n_ctx, self.n_q_heads, self.n_kv_heads, self.head_dim, self.dtype,
                         ctypes.cast(self._len, ctypes.POINTER(ctypes.c_int32)),
                         ctypes.cast(self._k, ctypes.POINTER(ctypes.c_void_p)),
                         ctypes.cast(self._v, ctypes.POINTER(ctypes.c_void_p)) if self._v is not None else None)

    @property
    def total_len(self) -> int:
        return sum(self.lens)


def samkv_peak_mfma_bf16(sink: torch.Tensor, n_blocks: int, iters: int) -> int:
    """Launches the pure-MFMA micro-kernel; returns the flop of the launch."""
    _check(_lib.samkv_peak_mfma_bf16(_ptr(sink), n_blocks, iters, _stream()), "samkv_peak_mfma_bf16")
    return n_blocks * 4 * iters * 16 * 32768


def samkv_peak_mfma_bf16_data(sink: torch.Tensor, n_blocks: int, iters: int, pattern: int) -> int:
    """The same with an operand pattern (0 small integers, 1 zeros, 2 random full mantissas); returns the flop."""
    _check(_lib.samkv_peak_mfma_bf16_data(_ptr(sink), n_blocks, iters, pattern, _stream()), "samkv_peak_mfma_bf16_data")
    return n_blocks * 4 * iters * 16 * 32768


def samkv_peak_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Launches the plain copy micro-kernel; returns the bytes moved (read + written)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(_lib.samkv_peak_copy(_ptr(src), _ptr(dst), nbytes, _stream()), "samkv_peak_copy")
    return 2 * nbytes


def samkv_peak_read(src: torch.Tensor, sink: torch.Tensor) -> int:
    """Launches the plain read micro-kernel; returns the bytes read."""
    nbytes = src.numel() * src.element_size()
    _check(_lib.samkv_peak_read(_ptr(src), nbytes, _ptr(sink), _stream()), "samkv_peak_read")
    return nbytes


def samkv_kept_count(length: int, ratio: float) -> int:
    return int(_lib.samkv_kept_count(length, ratio))


def samkv_workspace_bytes(n_ctx: int, n_q_heads: int, n_kv_heads: int, head_dim: int, n_q_tok: int,
                          m_total: int) -> int:
    return int(_lib.samkv_workspace_bytes(n_ctx, n_q_heads, n_kv_heads, head_dim, n_q_tok, m_total))


def samkv_score(caches: Caches, q_tok: torch.Tensor, q_loc: Optional[torch.Tensor], scores: torch.Tensor,
                ws: torch.Tensor) -> None:
    """scores [Hkv, sum L] float32 <- inner products of every key with its document's personalized query."""
    n_q_tok = int(q_tok.shape[1])
    w_loc = int(q_loc.shape[2]) if q_loc is not None else 0
    assert scores.dtype == torch.float32 and tuple(scores.shape) == (caches.n_kv_heads, caches.total_len)
    _check(_lib.samkv_score(ctypes.byref(caches.c), _ptr(q_tok), n_q_tok, _ptr(q_loc), w_loc, _ptr(scores),
                            _ptr(ws), ws.numel() * ws.element_size(), _stream()), "samkv_score")


def samkv_score_noalloc(caches: Caches, q_tok: torch.Tensor, q_loc: Optional[torch.Tensor], scores: torch.Tensor) -> None:
    """samkv_score without a workspace argument: the library's own fixed scratch area serves (sizes beyond it raise)."""
    n_q_tok = int(q_tok.shape[1])
    w_loc = int(q_loc.shape[2]) if q_loc is not None else 0
    assert scores.dtype == torch.float32 and tuple(scores.shape) == (caches.n_kv_heads, caches.total_len)
    _check(_lib.samkv_score_noalloc(ctypes.byref(caches.c), _ptr(q_tok), n_q_tok, _ptr(q_loc), w_loc, _ptr(scores),
                                    _stream()), "samkv_score_noalloc")


def samkv_score_select(caches: Caches, q_tok: torch.Tensor, q_loc: Optional[torch.Tensor], ratio: float, n_sink: int,
                       n_local: int, scores: Optional[torch.Tensor], idx: torch.Tensor,
                       cu_k_dev: Optional[torch.Tensor], ws: torch.Tensor) -> List[int]:
    """Score and selection in one pass over K; `scores` may be None.  Returns the host prefix sums cu_k."""
    n_q_tok = int(q_tok.shape[1])
    w_loc = int(q_loc.shape[2]) if q_loc is not None else 0
    assert scores is None or (scores.dtype == torch.float32 and tuple(scores.shape) == (caches.n_kv_heads, caches.total_len))
    assert idx.dtype == torch.int32
    assert tuple(idx.shape) == (caches.n_kv_heads, sum(samkv_kept_count(n, ratio) for n in caches.lens))
    cu_k_host = (ctypes.c_int32 * (caches.n_ctx + 1))()
    _check(_lib.samkv_score_select(ctypes.byref(caches.c), _ptr(q_tok), n_q_tok, _ptr(q_loc), w_loc, ratio, n_sink,
                                   n_local, _ptr(scores), _ptr(idx), _ptr(cu_k_dev), cu_k_host, _ptr(ws),
                                   ws.numel() * ws.element_size(), _stream()), "samkv_score_select")
    return list(cu_k_host)


def samkv_score_select_gather(caches: Caches, q_tok: torch.Tensor, q_loc: Optional[torch.Tensor], ratio: float,
                              n_sink: int, n_local: int, scores: Optional[torch.Tensor], idx: torch.Tensor,
                              cu_k_dev: Optional[torch.Tensor], k_c: torch.Tensor, v_c: torch.Tensor,
                              ws: torch.Tensor) -> List[int]:
    """samkv_score_select and samkv_gather in one call; returns the host prefix sums cu_k."""
    n_q_tok = int(q_tok.shape[1])
    w_loc = int(q_loc.shape[2]) if q_loc is not None else 0
    m = sum(samkv_kept_count(n, ratio) for n in caches.lens)
    assert scores is None or (scores.dtype == torch.float32 and tuple(scores.shape) == (caches.n_kv_heads, caches.total_len))
    assert idx.dtype == torch.int32 and tuple(idx.shape) == (caches.n_kv_heads, m)
    for x in (k_c, v_c):
        assert x.is_contiguous() and tuple(x.shape) == (caches.n_kv_heads, m, caches.head_dim) and x.dtype == q_tok.dtype
    cu_k_host = (ctypes.c_int32 * (caches.n_ctx + 1))()
    _check(_lib.samkv_score_select_gather(ctypes.byref(caches.c), _ptr(q_tok), n_q_tok, _ptr(q_loc), w_loc, ratio, n_sink,
                                          n_local, _ptr(scores), _ptr(idx), _ptr(cu_k_dev), cu_k_host, _ptr(k_c),
                                          _ptr(v_c), _ptr(ws), ws.numel() * ws.element_size(), _stream()),
           "samkv_score_select_gather")
    return list(cu_k_host)


def samkv_topk_select(scores: torch.Tensor, caches: Caches, ratio: float, n_sink: int, n_local: int,
                      idx: torch.Tensor, cu_k_dev: Optional[torch.Tensor], ws: Optional[torch.Tensor] = None
                      ) -> List[int]:
    """idx [Hkv, M] int32 <- kept positions; returns the host prefix sums cu_k (length n_ctx + 1)."""
    cu_k_host = (ctypes.c_int32 * (caches.n_ctx + 1))()
    assert idx.dtype == torch.int32
    assert tuple(idx.shape) == (caches.n_kv_heads, sum(samkv_kept_count(n, ratio) for n in caches.lens))
    _check(_lib.samkv_topk_select(_ptr(scores), ctypes.byref(caches.c), ratio, n_sink, n_local, _ptr(idx),
                                  _ptr(cu_k_dev), cu_k_host, _ptr(ws),
                                  ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
           "samkv_topk_select")
    return list(cu_k_host)


def samkv_kept_count_mid(length: int, p: float, n_sink: int, n_local: int) -> int:
    return int(_lib.samkv_kept_count_mid(length, p, n_sink, n_local))


def samkv_top_p(s_anc, s_max, s_min) -> List[float]:
    """Eq. 2 and Eq. 3 on host arrays [n_layers][n_ctx] -> P_i per document."""
    n_layers, n_ctx = len(s_anc), len(s_anc[0])
    flat = lambda a: (ctypes.c_float * (n_layers * n_ctx))(*[float(x) for row in a for x in row])
    out = (ctypes.c_float * n_ctx)()
    _check(_lib.samkv_top_p(flat(s_anc), flat(s_max), flat(s_min), n_layers, n_ctx, out), "samkv_top_p")
    return list(out)


def samkv_topk_select_v(scores: torch.Tensor, caches: Caches, p: Sequence[float], n_sink: int, n_local: int,
                        idx: torch.Tensor, cu_k_dev: Optional[torch.Tensor]) -> List[int]:
    """Selection with one middle-segment share per document; returns the host prefix sums cu_k."""
    cu_k_host = (ctypes.c_int32 * (caches.n_ctx + 1))()
    pp = (ctypes.c_float * caches.n_ctx)(*[float(x) for x in p])
    assert idx.dtype == torch.int32 and tuple(idx.shape) == (
        caches.n_kv_heads, sum(max(0, samkv_kept_count_mid(n, pi, n_sink, n_local)) for n, pi in zip(caches.lens, p)))
    _check(_lib.samkv_topk_select_v(_ptr(scores), ctypes.byref(caches.c), pp, n_sink, n_local, _ptr(idx),
                                    _ptr(cu_k_dev), cu_k_host, None, 0, _stream()), "samkv_topk_select_v")
    return list(cu_k_host)


def samkv_gather_v(caches: Caches, idx: torch.Tensor, cu_k: Sequence[int], k_c: torch.Tensor, v_c: torch.Tensor) -> None:
    cu = (ctypes.c_int32 * (caches.n_ctx + 1))(*[int(x) for x in cu_k])
    _check(_lib.samkv_gather_v(ctypes.byref(caches.c), _ptr(idx), cu, _ptr(k_c), _ptr(v_c), _stream()), "samkv_gather_v")


def samkv_block_scores(scores: torch.Tensor, caches: Caches, block: int, bscores: torch.Tensor) -> None:
    """bscores [Hkv, sum ceil(L_i / block)] float32 <- mean token score of every block."""
    assert scores.dtype == torch.float32 and bscores.dtype == torch.float32
    assert tuple(bscores.shape) == (caches.n_kv_heads, sum(-(-n // block) for n in caches.lens))
    _check(_lib.samkv_block_scores(_ptr(scores), ctypes.byref(caches.c), block, _ptr(bscores), _stream()),
           "samkv_block_scores")


def samkv_block_workspace_bytes(caches: Caches, block: int) -> int:
    return int(_lib.samkv_block_workspace_bytes(ctypes.byref(caches.c), block))


def samkv_block_select_count(caches: Caches, block: int, p: Sequence[float], n_init_blocks: int,
                             n_local_blocks: int) -> int:
    pp = (ctypes.c_float * caches.n_ctx)(*[float(x) for x in p])
    return int(_lib.samkv_block_select_count(ctypes.byref(caches.c), block, pp, n_init_blocks, n_local_blocks))


def samkv_block_select(bscores: torch.Tensor, caches: Caches, block: int, p: Sequence[float], n_init_blocks: int,
                       n_local_blocks: int, idx: torch.Tensor, cu_k_dev: Optional[torch.Tensor],
                       ws: torch.Tensor) -> List[int]:
    """idx [Hkv, M] int32 <- token positions of the kept blocks; returns the host prefix sums of kept tokens."""
    cu_k_host = (ctypes.c_int32 * (caches.n_ctx + 1))()
    pp = (ctypes.c_float * caches.n_ctx)(*[float(x) for x in p])
    assert idx.dtype == torch.int32 and bscores.dtype == torch.float32
    m = samkv_block_select_count(caches, block, p, n_init_blocks, n_local_blocks)
    assert m == 0 or tuple(idx.shape) == (caches.n_kv_heads, m), "idx must be [Hkv, samkv_block_select_count(...)]"
    _check(_lib.samkv_block_select(_ptr(bscores), ctypes.byref(caches.c), block, pp, n_init_blocks, n_local_blocks,
                                   _ptr(idx), _ptr(cu_k_dev), cu_k_host, _ptr(ws), ws.numel() * ws.element_size(),
                                   _stream()), "samkv_block_select")
    return list(cu_k_host)


def samkv_block_filter_count(caches: Caches, block: int, p: Sequence[float], n_init_blocks: int,
                             n_local_blocks: int) -> int:
    pp = (ctypes.c_float * caches.n_ctx)(*[float(x) for x in p])
    return int(_lib.samkv_block_filter_count(ctypes.byref(caches.c), block, pp, n_init_blocks, n_local_blocks))


def samkv_block_select_filter(bscores: torch.Tensor, caches: Caches, block: int, p: Sequence[float], n_init_blocks: int,
                              n_local_blocks: int, gidx: torch.Tensor, ws: torch.Tensor) -> None:
    """gidx [Hkv, M] int32 <- global token positions kept after the cross-document filter."""
    pp = (ctypes.c_float * caches.n_ctx)(*[float(x) for x in p])
    assert gidx.dtype == torch.int32 and bscores.dtype == torch.float32
    assert gidx.shape[1] == samkv_block_filter_count(caches, block, p, n_init_blocks, n_local_blocks)
    _check(_lib.samkv_block_select_filter(_ptr(bscores), ctypes.byref(caches.c), block, pp, n_init_blocks,
                                          n_local_blocks, _ptr(gidx), _ptr(ws), ws.numel() * ws.element_size(),
                                          _stream()), "samkv_block_select_filter")


def samkv_gather_g(caches: Caches, gidx: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor) -> None:
    assert gidx.dtype == torch.int32 and tuple(k_c.shape) == (caches.n_kv_heads, gidx.shape[1], caches.head_dim)
    _check(_lib.samkv_gather_g(ctypes.byref(caches.c), _ptr(gidx), int(gidx.shape[1]), _ptr(k_c), _ptr(v_c), _stream()),
           "samkv_gather_g")


def samkv_gather_q_g(caches: Caches, q_cache: Sequence[torch.Tensor], gidx: torch.Tensor, q_rec: torch.Tensor) -> None:
    assert len(q_cache) == caches.n_ctx and gidx.dtype == torch.int32
    assert tuple(q_rec.shape) == (caches.n_q_heads, gidx.shape[1], caches.head_dim)
    ptrs = (ctypes.c_void_p * caches.n_ctx)(*[t.data_ptr() for t in q_cache])
    _check(_lib.samkv_gather_q_g(ctypes.byref(caches.c), ptrs, _ptr(gidx), int(gidx.shape[1]), _ptr(q_rec), _stream()),
           "samkv_gather_q_g")


def samkv_gather_q_v(caches: Caches, q_cache: Sequence[torch.Tensor], idx: torch.Tensor, cu_k: Sequence[int],
                     q_rec: torch.Tensor) -> None:
    assert len(q_cache) == caches.n_ctx and idx.dtype == torch.int32
    ptrs = (ctypes.c_void_p * caches.n_ctx)(*[t.data_ptr() for t in q_cache])
    cu = (ctypes.c_int32 * (caches.n_ctx + 1))(*[int(x) for x in cu_k])
    _check(_lib.samkv_gather_q_v(ctypes.byref(caches.c), ptrs, _ptr(idx), cu, _ptr(q_rec), _stream()),
           "samkv_gather_q_v")


def samkv_gather(caches: Caches, idx: torch.Tensor, ratio: float, k_c: torch.Tensor, v_c: torch.Tensor) -> None:
    """k_c, v_c [Hkv, M, d] <- kept rows of every document, concatenated."""
    assert idx.dtype == torch.int32 and k_c.dtype == caches.k[0].dtype and v_c.dtype == caches.k[0].dtype
    _check(_lib.samkv_gather(ctypes.byref(caches.c), _ptr(idx), ratio, _ptr(k_c), _ptr(v_c), _stream()),
           "samkv_gather")


def samkv_gather_q(caches: Caches, q_cache: Sequence[torch.Tensor], idx: torch.Tensor, ratio: float,
                   q_rec: torch.Tensor) -> None:
    """q_rec [Hq, M, d] <- rows of the per-document Q caches ([Hq, L_i, d]) at the kept positions of each head's KV head."""
    assert len(q_cache) == caches.n_ctx and idx.dtype == torch.int32
    for t, L in zip(q_cache, caches.lens):
        assert t.is_cuda and t.is_contiguous() and tuple(t.shape) == (caches.n_q_heads, L, caches.head_dim)
        assert t.dtype == caches.k[0].dtype
    ptrs = (ctypes.c_void_p * caches.n_ctx)(*[t.data_ptr() for t in q_cache])
    _check(_lib.samkv_gather_q(ctypes.byref(caches.c), ptrs, _ptr(idx), ratio, _ptr(q_rec), _stream()), "samkv_gather_q")


def samkv_recompute_attn(q_rec: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor, scale: float,
                         out: torch.Tensor, lse: torch.Tensor, ws: Optional[torch.Tensor] = None) -> None:
    """out [Hq, M, d], lse [Hq, M] float32 <- causal attention of the kept tokens over the compacted cache."""
    hq, m, d = q_rec.shape
    hkv = k_c.shape[0]
    assert k_c.shape == (hkv, m, d) and v_c.shape == (hkv, m, d) and out.dtype == lse.dtype == torch.float32
    assert tuple(out.shape) == (hq, m, d) and tuple(lse.shape) == (hq, m)
    _check(_lib.samkv_recompute_attn(_ptr(q_rec), _ptr(k_c), _ptr(v_c), m, hq, hkv, d, _dtype_code(q_rec.dtype),
                                     scale, _ptr(out), _ptr(lse), _ptr(ws),
                                     ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
           "samkv_recompute_attn")


def samkv_query_attn(q_tok: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor, scale: float, out: torch.Tensor,
                     lse: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    """out [Hq, Lq, d], lse [Hq, Lq] float32 <- attention of the query tokens over the compacted cache."""
    hq, lq, d = q_tok.shape
    hkv, m, _ = k_c.shape
    assert v_c.shape == k_c.shape and out.dtype == lse.dtype == torch.float32
    assert tuple(out.shape) == (hq, lq, d) and tuple(lse.shape) == (hq, lq)
    _check(_lib.samkv_query_attn(_ptr(q_tok), lq, _ptr(k_c), _ptr(v_c), m, hq, hkv, d, _dtype_code(q_tok.dtype),
                                 scale, _ptr(out), _ptr(lse), _ptr(ws),
                                 ws.numel() * ws.element_size() if ws is not None else 0, _stream()),
           "samkv_query_attn")


def samkv_recompute_query_attn(q_rec: torch.Tensor, q_tok: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor,
                               scale: float, rec_out: torch.Tensor, rec_lse: torch.Tensor, q_out: torch.Tensor,
                               q_lse: torch.Tensor, ws: Optional[torch.Tensor]) -> None:
    """samkv_recompute_attn and samkv_query_attn over the same compacted cache in one call (V prepared once)."""
    hq, m, d = q_rec.shape
    lq = int(q_tok.shape[1])
    hkv = k_c.shape[0]
    assert k_c.shape == (hkv, m, d) and v_c.shape == (hkv, m, d) and tuple(q_tok.shape) == (hq, lq, d)
    assert tuple(rec_out.shape) == (hq, m, d) and tuple(rec_lse.shape) == (hq, m)
    assert tuple(q_out.shape) == (hq, lq, d) and tuple(q_lse.shape) == (hq, lq)
    for x in (rec_out, rec_lse, q_out, q_lse):
        assert x.dtype == torch.float32
    _check(_lib.samkv_recompute_query_attn(_ptr(q_rec), _ptr(q_tok), lq, _ptr(k_c), _ptr(v_c), m, hq, hkv, d,
                                           _dtype_code(q_rec.dtype), scale, _ptr(rec_out), _ptr(rec_lse), _ptr(q_out),
                                           _ptr(q_lse), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                           _stream()), "samkv_recompute_query_attn")


def samkv_query_attn_self(q_tok: torch.Tensor, k_c: torch.Tensor, v_c: torch.Tensor, k_self: torch.Tensor,
                          v_self: torch.Tensor, scale: float, out: torch.Tensor, lse: torch.Tensor,
                          ws: torch.Tensor) -> None:
    """As samkv_query_attn, with the query tokens' own K/V [Hkv, Lq, d] appended causally."""
    hq, lq, d = q_tok.shape
    hkv, m, _ = k_c.shape
    assert tuple(k_self.shape) == (hkv, lq, d) and v_self.shape == k_self.shape and v_c.shape == k_c.shape
    assert tuple(out.shape) == (hq, lq, d) and tuple(lse.shape) == (hq, lq) and out.dtype == lse.dtype == torch.float32
    _check(_lib.samkv_query_attn_self(_ptr(q_tok), lq, _ptr(k_c), _ptr(v_c), m, _ptr(k_self), _ptr(v_self), hq, hkv, d,
                                      _dtype_code(q_tok.dtype), scale, _ptr(out), _ptr(lse), _ptr(ws),
                                      ws.numel() * ws.element_size(), _stream()), "samkv_query_attn_self")


def samkv_kv_update(k_c: torch.Tensor, v_c: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, mode: int) -> None:
    """k_c, v_c [Hkv, M, d] <- overwrite (mode 0) or cosine-weighted fusion (mode 1, Eq. 4) with k_new, v_new."""
    hkv, m, d = k_c.shape
    for t in (v_c, k_new, v_new):
        assert t.shape == k_c.shape and t.dtype == k_c.dtype
    _check(_lib.samkv_kv_update(_ptr(k_c), _ptr(v_c), _ptr(k_new), _ptr(v_new), m, hkv, d, _dtype_code(k_c.dtype),
                                mode, _stream()), "samkv_kv_update")


# ------------------------------------------------------------------------------------------------
@dataclass
class LayerBuffers:
    """Device buffers of one pass of the hot path over one layer (allocated once, reused)."""

    scores: torch.Tensor
    idx: torch.Tensor
    cu_k_dev: torch.Tensor
    k_c: torch.Tensor
    v_c: torch.Tensor
    rec_out: torch.Tensor
    rec_lse: torch.Tensor
    q_out: torch.Tensor
    q_lse: torch.Tensor
    ws: torch.Tensor
    cu_k: List[int]


def alloc_layer_buffers(caches: Caches, n_q_tok: int, ratio: float) -> LayerBuffers:
    dev = caches.k[0].device
    ks = [samkv_kept_count(L, ratio) for L in caches.lens]
    m = sum(ks)
    hq, hkv, d = caches.n_q_heads, caches.n_kv_heads, caches.head_dim
    dt = caches.k[0].dtype
    ws_bytes = samkv_workspace_bytes(caches.n_ctx, hq, hkv, d, n_q_tok, m)
    f32 = dict(device=dev, dtype=torch.float32)
    return LayerBuffers(
        scores=torch.empty((hkv, caches.total_len), **f32),
        idx=torch.empty((hkv, m), device=dev, dtype=torch.int32),
        cu_k_dev=torch.empty((caches.n_ctx + 1,), device=dev, dtype=torch.int32),
        k_c=torch.empty((hkv, m, d), device=dev, dtype=dt), v_c=torch.empty((hkv, m, d), device=dev, dtype=dt),
        rec_out=torch.empty((hq, m, d), **f32), rec_lse=torch.empty((hq, m), **f32),
        q_out=torch.empty((hq, n_q_tok, d), **f32), q_lse=torch.empty((hq, n_q_tok), **f32),
        ws=torch.empty((ws_bytes,), device=dev, dtype=torch.uint8),
        cu_k=[0] + list(__import__("itertools").accumulate(ks)),
    )


def hot_path(caches: Caches, q_tok: torch.Tensor, q_loc: Optional[torch.Tensor], q_rec: torch.Tensor,
             ratio: float, scale: float, buf: LayerBuffers, n_sink: int = 0, n_local: int = 0,
             fused: bool = True) -> None:
    """One pass of the whole hot path of a layer: score, select, gather, recompute, query attention.  `fused`
    scores, selects and compacts in one call and runs both attentions in one call (same kept positions, same bits);
    otherwise the five separate calls."""
    if fused:
        samkv_score_select_gather(caches, q_tok, q_loc, ratio, n_sink, n_local, buf.scores, buf.idx, buf.cu_k_dev,
                                  buf.k_c, buf.v_c, buf.ws)
    else:
        samkv_score(caches, q_tok, q_loc, buf.scores, buf.ws)
        samkv_topk_select(buf.scores, caches, ratio, n_sink, n_local, buf.idx, buf.cu_k_dev, buf.ws)
        samkv_gather(caches, buf.idx, ratio, buf.k_c, buf.v_c)
    if fused:
        samkv_recompute_query_attn(q_rec, q_tok, buf.k_c, buf.v_c, scale, buf.rec_out, buf.rec_lse, buf.q_out, buf.q_lse,
                                   buf.ws)
    else:
        samkv_recompute_attn(q_rec, buf.k_c, buf.v_c, scale, buf.rec_out, buf.rec_lse, buf.ws)
        samkv_query_attn(q_tok, buf.k_c, buf.v_c, scale, buf.q_out, buf.q_lse, buf.ws)
