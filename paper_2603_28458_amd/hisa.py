"""ctypes binding of libhisa.so (C ABI in include/hisa.h).  Argument marshalling only: every
step of the indexer runs in the HIP kernels.  PyTorch supplies device memory and the stream.

The functions carry the names of the C entry points.  There is no CPU fallback: if the compiled
library is missing, the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

HISA_F32, HISA_BF16, HISA_FP8_E4M3 = 0, 1, 2
OP_POOL, OP_BLOCK_SCORE_TOPK, OP_TOKEN_REFINE_TOPK, OP_FLAT_TOPK = 0, 1, 2, 3
DTYPE_CODE = {"f32": HISA_F32, "bf16": HISA_BF16, "fp8_e4m3": HISA_FP8_E4M3}
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libhisa.so")

EXPORTS = ["hisa_pool_blocks", "hisa_pool_append", "hisa_block_score_topk", "hisa_token_refine_topk",
           "hisa_block_sparse_tokens", "hisa_index_iou", "dsa_flat_indexer_topk", "hisa_workspace_bytes",
           "hisa_status_string", "hisa_version", "hisa_probe_copy", "hisa_probe_mfma", "hisa_probe_mfma_fp8", "hisa_probe_mfma_toggling", "hisa_indexer_topk", "hisa_pool_blocks_max",
           "hisa_token_refine_topk_static"]
STATIC_SCRATCH_BYTES = 16 << 20


class HisaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class _Keys(C.Structure):
    _fields_ = [("k", C.c_void_p), ("k_scale", C.c_void_p), ("seq_len", C.c_void_p),
                ("n_seq", C.c_int32), ("s_max", C.c_int32), ("d", C.c_int32), ("k_dtype", C.c_int32)]


class _Queries(C.Structure):
    _fields_ = [("q", C.c_void_p), ("w", C.c_void_p), ("q_seq", C.c_void_p), ("q_pos", C.c_void_p),
                ("q_lo", C.c_void_p), ("T", C.c_int32), ("H", C.c_int32), ("q_pos0", C.c_int32),
                ("q_dtype", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2603_28458_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               f"`python -m paper_2603_28458_amd.build` (there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.hisa_pool_blocks.argtypes = [C.POINTER(_Keys), i32, i32, i32, vp, i32, vp]
        L.hisa_pool_blocks.restype = C.c_int
        L.hisa_pool_blocks_max.argtypes = [C.POINTER(_Keys), i32, i32, i32, vp, i32, vp]
        L.hisa_pool_blocks_max.restype = C.c_int
        L.hisa_pool_append.argtypes = [C.POINTER(_Keys), i32, vp, i32, vp, i32, vp]
        L.hisa_pool_append.restype = C.c_int
        L.hisa_block_sparse_tokens.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), i32, i32, vp, vp, vp]
        L.hisa_block_sparse_tokens.restype = C.c_int
        L.hisa_index_iou.argtypes = [vp, vp, i32, i32, vp, vp]
        L.hisa_index_iou.restype = C.c_int
        L.hisa_block_score_topk.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), vp, i32, i32, i32,
                                            vp, vp, vp, sz, vp]
        L.hisa_block_score_topk.restype = C.c_int
        L.hisa_token_refine_topk.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), i32, i32, vp, i32,
                                             vp, vp, vp, vp, sz, vp]
        L.hisa_token_refine_topk.restype = C.c_int
        L.hisa_token_refine_topk_static.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), i32, i32, vp, i32,
                                                    vp, vp, vp]
        L.hisa_token_refine_topk_static.restype = C.c_int
        L.dsa_flat_indexer_topk.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), i32, vp, vp, vp,
                                            sz, vp]
        L.dsa_flat_indexer_topk.restype = C.c_int
        L.hisa_workspace_bytes.argtypes = [C.c_int, C.POINTER(_Queries), C.POINTER(_Keys), i32, i32,
                                           i32, i32]
        L.hisa_workspace_bytes.restype = sz
        L.hisa_indexer_topk.argtypes = [C.POINTER(_Queries), C.POINTER(_Keys), vp, i32, i32, i32, i32, vp, vp,
                                        vp, vp]
        L.hisa_indexer_topk.restype = C.c_int
        L.hisa_probe_copy.argtypes = [vp, vp, sz, vp]
        L.hisa_probe_copy.restype = C.c_int
        L.hisa_probe_mfma.argtypes = [vp, i32, C.POINTER(C.c_double), vp]
        L.hisa_probe_mfma.restype = C.c_int
        L.hisa_probe_mfma_fp8.argtypes = [vp, i32, C.POINTER(C.c_double), vp]
        L.hisa_probe_mfma_fp8.restype = C.c_int
        L.hisa_probe_mfma_toggling.argtypes = [vp, i32, i32, C.POINTER(C.c_double), vp]
        L.hisa_probe_mfma_toggling.restype = C.c_int
        L.hisa_status_string.argtypes = [C.c_int]
        L.hisa_status_string.restype = C.c_char_p
        L.hisa_version.argtypes = []
        L.hisa_version.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hisa_status_string(int(status)).decode()


def version() -> str:
    return lib().hisa_version().decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


@dataclass
class Keys:
    """Token-level indexing keys: k [n_seq, s_max, d] (float32 / bfloat16 / uint8 or float8 codes),
    k_scale [n_seq, s_max] float32 for fp8, seq_len [n_seq] int32; all on the GPU."""
    k: Optional[torch.Tensor]
    seq_len: torch.Tensor
    dtype: int
    k_scale: Optional[torch.Tensor] = None
    n_seq: int = 0
    s_max: int = 0
    d: int = 0

    def __post_init__(self):
        if self.k is not None:
            self.n_seq, self.s_max, self.d = self.k.shape

    def c(self) -> _Keys:
        return _Keys(_ptr(self.k), _ptr(self.k_scale), _ptr(self.seq_len), self.n_seq, self.s_max,
                     self.d, self.dtype)


@dataclass
class Queries:
    """Indexing queries q [T, H, d] (float32 / bfloat16), gates w [T, H] float32, optional
    q_seq / q_pos / q_lo [T] int32; all on the GPU."""
    q: torch.Tensor
    w: torch.Tensor
    dtype: int
    q_seq: Optional[torch.Tensor] = None
    q_pos: Optional[torch.Tensor] = None
    q_pos0: int = 0
    q_lo: Optional[torch.Tensor] = None

    @property
    def T(self) -> int:
        return self.q.shape[0]

    @property
    def H(self) -> int:
        return self.q.shape[1]

    def c(self) -> _Queries:
        return _Queries(_ptr(self.q), _ptr(self.w), _ptr(self.q_seq), _ptr(self.q_pos), _ptr(self.q_lo),
                        self.T, self.H, self.q_pos0, self.dtype)


def _check(status: int, where: str):
    if status != 0:
        raise HisaError(status, where)


def hisa_workspace_bytes(op: int, queries: Queries, keys: Keys, B: int = 1, m: int = 0, k: int = 0,
                         want_scores: bool = False) -> int:
    qc, kc = queries.c(), keys.c()
    return int(lib().hisa_workspace_bytes(op, C.byref(qc), C.byref(kc), B, m, k, int(want_scores)))


def _ws(ws: Optional[torch.Tensor], nbytes: int, device) -> Optional[torch.Tensor]:
    if ws is not None or nbytes == 0:
        return ws
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


_POOLED_TORCH = {HISA_F32: torch.float32, HISA_BF16: torch.bfloat16}


def hisa_pool_blocks(keys: Keys, B: int, pooled: Optional[torch.Tensor] = None,
                     pooled_dtype: int = HISA_BF16, blk_begin: int = 0, blk_end: Optional[int] = None,
                     stream=None, max_pool: bool = False) -> torch.Tensor:
    """Eq. 4: pooled [n_seq, s_max / B, d] (max_pool: hisa_pool_blocks_max, the maximum instead of the mean)."""
    M = keys.s_max // B
    if pooled is None:
        pooled = torch.zeros((keys.n_seq, M, keys.d), dtype=_POOLED_TORCH[pooled_dtype],
                             device=keys.k.device)
    kc = keys.c()
    fn = lib().hisa_pool_blocks_max if max_pool else lib().hisa_pool_blocks
    st = fn(C.byref(kc), B, blk_begin, M if blk_end is None else blk_end, _ptr(pooled), pooled_dtype,
            _stream(stream))
    _check(st, "hisa_pool_blocks_max" if max_pool else "hisa_pool_blocks")
    return pooled


def hisa_pool_blocks_max(keys: Keys, B: int, pooled: Optional[torch.Tensor] = None, pooled_dtype: int = HISA_BF16,
                         blk_begin: int = 0, blk_end: Optional[int] = None, stream=None) -> torch.Tensor:
    """Eq. 4 with Pool = per-dimension maximum."""
    return hisa_pool_blocks(keys, B, pooled, pooled_dtype, blk_begin, blk_end, stream, max_pool=True)


def hisa_pool_append(keys: Keys, B: int, prev_len: torch.Tensor, max_new_tokens: int, pooled: torch.Tensor,
                     pooled_dtype: int = HISA_BF16, stream=None) -> torch.Tensor:
    """Section 4.1, incremental pooled cache: re-pools the blocks that grew since prev_len."""
    kc = keys.c()
    st = lib().hisa_pool_append(C.byref(kc), B, _ptr(prev_len), max_new_tokens, _ptr(pooled), pooled_dtype,
                                _stream(stream))
    _check(st, "hisa_pool_append")
    return pooled


def hisa_block_sparse_tokens(queries: Queries, keys: Keys, B: int, m: int, block_idx: torch.Tensor,
                             tokens: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Block-Sparse baseline (Section 5): tokens [T, m*B] int32, -1 where not visible."""
    if tokens is None:
        tokens = torch.empty((queries.T, m * B), dtype=torch.int32, device=block_idx.device)
    qc, kc = queries.c(), keys.c()
    st = lib().hisa_block_sparse_tokens(C.byref(qc), C.byref(kc), B, m, _ptr(block_idx), _ptr(tokens),
                                        _stream(stream))
    _check(st, "hisa_block_sparse_tokens")
    return tokens


def hisa_index_iou(a_idx: torch.Tensor, b_idx: torch.Tensor, iou: Optional[torch.Tensor] = None,
                   stream=None) -> torch.Tensor:
    """Eq. 12 per row of two [T, k] index tensors (ascending rows, -1 padding)."""
    T, k = a_idx.shape
    assert b_idx.shape == a_idx.shape
    if iou is None:
        iou = torch.empty((T,), dtype=torch.float32, device=a_idx.device)
    st = lib().hisa_index_iou(_ptr(a_idx), _ptr(b_idx), T, k, _ptr(iou), _stream(stream))
    _check(st, "hisa_index_iou")
    return iou


def hisa_block_score_topk(queries: Queries, keys: Keys, pooled: torch.Tensor, pooled_dtype: int, B: int,
                          m: int, block_idx: Optional[torch.Tensor] = None,
                          block_scores: Optional[torch.Tensor] = None, want_scores: bool = False,
                          ws: Optional[torch.Tensor] = None, stream=None):
    """Stage 1 (Eqs. 5-6).  Returns (block_idx [T, m] int32, block_scores [T, s_max/B] or None)."""
    dev = queries.q.device
    T, M = queries.T, keys.s_max // B
    if block_idx is None:
        block_idx = torch.empty((T, m), dtype=torch.int32, device=dev)
    if want_scores and block_scores is None:
        block_scores = torch.empty((T, M), dtype=torch.float32, device=dev)
    ws = _ws(ws, hisa_workspace_bytes(OP_BLOCK_SCORE_TOPK, queries, keys, B, m, 0,
                                      block_scores is not None), dev)
    qc, kc = queries.c(), keys.c()
    st = lib().hisa_block_score_topk(C.byref(qc), C.byref(kc), _ptr(pooled), pooled_dtype, B, m,
                                     _ptr(block_idx), _ptr(block_scores), _ptr(ws),
                                     0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hisa_block_score_topk")
    return block_idx, block_scores


def hisa_token_refine_topk(queries: Queries, keys: Keys, B: int, m: int, block_idx: torch.Tensor, k: int,
                           topk_idx: Optional[torch.Tensor] = None,
                           topk_scores: Optional[torch.Tensor] = None,
                           cand_scores: Optional[torch.Tensor] = None, want_topk_scores: bool = False,
                           want_cand_scores: bool = False, ws: Optional[torch.Tensor] = None, stream=None):
    """Stage 2 (Eqs. 7-9).  Returns (topk_idx [T, k] int32, topk_scores or None, cand_scores or None)."""
    dev = queries.q.device
    T = queries.T
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    if want_topk_scores and topk_scores is None:
        topk_scores = torch.empty((T, k), dtype=torch.float32, device=dev)
    if want_cand_scores and cand_scores is None:
        cand_scores = torch.empty((T, m * B), dtype=torch.float32, device=dev)
    ws = _ws(ws, hisa_workspace_bytes(OP_TOKEN_REFINE_TOPK, queries, keys, B, m, k,
                                      cand_scores is not None), dev)
    qc, kc = queries.c(), keys.c()
    st = lib().hisa_token_refine_topk(C.byref(qc), C.byref(kc), B, m, _ptr(block_idx), k, _ptr(topk_idx),
                                      _ptr(topk_scores), _ptr(cand_scores), _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hisa_token_refine_topk")
    return topk_idx, topk_scores, cand_scores


def hisa_token_refine_topk_static(queries: Queries, keys: Keys, B: int, m: int, block_idx: torch.Tensor, k: int,
                                  topk_idx: torch.Tensor, topk_scores: Optional[torch.Tensor] = None,
                                  stream=None):
    """Stage 2 (Eqs. 7-9) through the library's static scratch array: nothing is allocated, here or
    in the library, so the outputs must be passed in.  Returns (topk_idx, topk_scores)."""
    qc, kc = queries.c(), keys.c()
    st = lib().hisa_token_refine_topk_static(C.byref(qc), C.byref(kc), B, m, _ptr(block_idx), k, _ptr(topk_idx),
                                             _ptr(topk_scores), _stream(stream))
    _check(st, "hisa_token_refine_topk_static")
    return topk_idx, topk_scores


def dsa_flat_indexer_topk(queries: Queries, keys: Keys, k: int, topk_idx: Optional[torch.Tensor] = None,
                          topk_scores: Optional[torch.Tensor] = None, want_topk_scores: bool = False,
                          ws: Optional[torch.Tensor] = None, stream=None):
    """Flat DSA indexer (Eqs. 1-2).  Returns (topk_idx [T, k] int32, topk_scores or None)."""
    dev = queries.q.device
    T = queries.T
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    if want_topk_scores and topk_scores is None:
        topk_scores = torch.empty((T, k), dtype=torch.float32, device=dev)
    ws = _ws(ws, hisa_workspace_bytes(OP_FLAT_TOPK, queries, keys, 1, 0, k), dev)
    qc, kc = queries.c(), keys.c()
    st = lib().dsa_flat_indexer_topk(C.byref(qc), C.byref(kc), k, _ptr(topk_idx), _ptr(topk_scores),
                                     _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "dsa_flat_indexer_topk")
    return topk_idx, topk_scores


def hisa_indexer_topk(queries: Queries, keys: Keys, pooled: torch.Tensor, pooled_dtype: int, B: int, m: int,
                      k: int, block_idx: Optional[torch.Tensor] = None, want_block_idx: bool = False,
                      topk_idx: Optional[torch.Tensor] = None, topk_scores: Optional[torch.Tensor] = None,
                      want_topk_scores: bool = False, stream=None):
    """Algorithm 1 in one launch.  Returns (block_idx or None, topk_idx, topk_scores or None)."""
    dev = queries.q.device
    T = queries.T
    if want_block_idx and block_idx is None:
        block_idx = torch.empty((T, m), dtype=torch.int32, device=dev)
    if topk_idx is None:
        topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    if want_topk_scores and topk_scores is None:
        topk_scores = torch.empty((T, k), dtype=torch.float32, device=dev)
    qc, kc = queries.c(), keys.c()
    st = lib().hisa_indexer_topk(C.byref(qc), C.byref(kc), _ptr(pooled), pooled_dtype, B, m, k, _ptr(block_idx),
                                 _ptr(topk_idx), _ptr(topk_scores), _stream(stream))
    _check(st, "hisa_indexer_topk")
    return block_idx, topk_idx, topk_scores


def hisa_probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> int:
    """Streaming copy probe; returns the bytes moved (read + written)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().hisa_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "hisa_probe_copy")
    return 2 * nbytes


def hisa_probe_mfma(out: torch.Tensor, iters: int, stream=None) -> float:
    """MFMA-only probe; `out` holds at least 512 * 256 floats; returns the flop count of the launch."""
    assert out.dtype == torch.float32 and out.numel() >= 512 * 256
    flop = C.c_double(0.0)
    _check(lib().hisa_probe_mfma(_ptr(out), iters, C.byref(flop), _stream(stream)), "hisa_probe_mfma")
    return flop.value


def hisa_probe_mfma_fp8(out: torch.Tensor, iters: int, stream=None) -> float:
    """The same probe on the fp8 MFMA (e4m3 x e4m3)."""
    assert out.dtype == torch.float32 and out.numel() >= 512 * 256
    flop = C.c_double(0.0)
    _check(lib().hisa_probe_mfma_fp8(_ptr(out), iters, C.byref(flop), _stream(stream)), "hisa_probe_mfma_fp8")
    return flop.value


def hisa_probe_mfma_toggling(out: torch.Tensor, iters: int, fp8: bool = False, stream=None) -> float:
    """Either MFMA probe on operands that differ per lane and per instruction (pseudo-random values)."""
    assert out.dtype == torch.float32 and out.numel() >= 512 * 256
    flop = C.c_double(0.0)
    _check(lib().hisa_probe_mfma_toggling(_ptr(out), iters, 1 if fp8 else 0, C.byref(flop), _stream(stream)),
           "hisa_probe_mfma_toggling")
    return flop.value


# ---------------------------------------------------------------- moving a workload to the GPU
def to_device(wl, device="cuda:0"):
    """(Queries, Keys) on the GPU from a workloads.Workload (host numpy bits): copies only."""
    import numpy as np

    def dev(a, view=None):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a))
        if view is not None:
            t = t.view(view)
        return t.to(device)

    kview = {"f32": None, "bf16": torch.bfloat16, "fp8_e4m3": None}[wl.k_dtype]
    kk = wl.keys.view(np.int16) if wl.k_dtype == "bf16" else wl.keys
    qq = wl.q.view(np.int16) if wl.q_dtype == "bf16" else wl.q
    keys = Keys(k=dev(kk, kview), seq_len=dev(wl.seq_len.astype(np.int32)), dtype=DTYPE_CODE[wl.k_dtype],
                k_scale=dev(wl.k_scale))
    queries = Queries(q=dev(qq, torch.bfloat16 if wl.q_dtype == "bf16" else None), w=dev(wl.w),
                      dtype=DTYPE_CODE[wl.q_dtype], q_seq=dev(wl.q_seq), q_pos=dev(wl.q_pos),
                      q_pos0=wl.q_pos0, q_lo=dev(getattr(wl, "q_lo", None)))
    return queries, keys
