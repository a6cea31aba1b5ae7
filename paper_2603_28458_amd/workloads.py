"""Seeded synthetic inputs for the HISA / DSA indexer (no indexer arithmetic lives here).

The paper evaluates on DeepSeek-V3.2 / GLM-5 indexer activations (Section 5); those models are
not available, so every tensor here is synthetic with the shapes of the paper's kernel benchmark
(Section 5.1: B=128, m=64, k=2048) and the value recipe below:

  keys     k_s = c_{floor(s/B)} + 0.5 * N(0,1),  centroids c_b ~ N(0,1)^d   (block-clustered)
  queries  q   ~ N(0,1)
  gates    w   ~ U(0,1), fp32
  needles  k_p = 3 * sqrt(1.25 d) * q_{t*,j*} / ||q_{t*,j*}||  at uniform random positions p,
           with t* uniform among the queries that can see p and j* a uniform head
  fp8      per-token scale = max_i |k_{s,i}| / 448, code = e4m3fn(k_s / scale), round-to-nearest-even

Both the CPU oracle and the HIP library receive the SAME stored bits.  Arrays are numpy:
fp32 as float32, bf16 as uint16 bit patterns, fp8 as uint8 codes.  Quantisation (a cast done by
torch's CPU conversion routines) is part of producing the inputs, not of the indexer.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

F32, BF16, FP8 = "f32", "bf16", "fp8_e4m3"
BASE_SEED = 20260328


_N_STREAMS = 16   # fixed, so the drawn values do not depend on the machine's core count


def _normal(ss: np.random.SeedSequence, shape) -> np.ndarray:
    """N(0,1) float32 array of `shape`, drawn as _N_STREAMS independent child streams over equal
    slices of the first axis (filled in parallel: numpy releases the GIL while drawing)."""
    from concurrent.futures import ThreadPoolExecutor
    out = np.empty(shape, dtype=np.float32)
    n = shape[0]
    bounds = [(i * n) // _N_STREAMS for i in range(_N_STREAMS + 1)]
    kids = ss.spawn(_N_STREAMS)

    def fill(i):
        lo, hi = bounds[i], bounds[i + 1]
        if hi > lo:
            np.random.default_rng(kids[i]).standard_normal(out=out[lo:hi], dtype=np.float32)

    with ThreadPoolExecutor(max_workers=min(_N_STREAMS, os.cpu_count() or 1)) as ex:
        list(ex.map(fill, range(_N_STREAMS)))
    return out


def _to_bf16_bits(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(b).view(np.int16)).view(torch.bfloat16)
    return t.to(torch.float32).numpy()


def _to_fp8(x: np.ndarray):
    """x [..., d] float32 -> (codes uint8 [..., d], scale float32 [...])."""
    amax = np.abs(x).max(axis=-1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = np.clip(x / scale[..., None], -448.0, 448.0).astype(np.float32)
    codes = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    return codes, scale


def _cast(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return _to_bf16_bits(x)
    raise ValueError(dtype)


def _as_f32(bits: np.ndarray, dtype: str) -> np.ndarray:
    return bits if dtype == F32 else _bf16_bits_to_f32(bits)


@dataclass
class Workload:
    name: str
    # shapes / hyper-parameters (paper notation: B block size, m block budget, k token budget)
    n_seq: int
    s_max: int
    T: int
    H: int
    d: int
    B: int
    m: int
    k: int
    q_dtype: str
    k_dtype: str
    pooled_dtype: str
    # tensors (numpy, raw stored bits)
    keys: np.ndarray = field(repr=False)            # [n_seq, s_max, d]
    k_scale: Optional[np.ndarray] = field(repr=False, default=None)  # [n_seq, s_max] f32 (fp8 only)
    seq_len: np.ndarray = field(repr=False, default=None)            # [n_seq] int32
    q: np.ndarray = field(repr=False, default=None)                  # [T, H, d]
    w: np.ndarray = field(repr=False, default=None)                  # [T, H] f32
    q_seq: Optional[np.ndarray] = field(repr=False, default=None)    # [T] int32 or None (all 0)
    q_pos: Optional[np.ndarray] = field(repr=False, default=None)    # [T] int32 or None
    q_pos0: int = 0                                                  # q_pos[t] = q_pos0 + t if q_pos is None
    q_lo: Optional[np.ndarray] = field(repr=False, default=None)     # [T] int32 first visible position, or None (0)
    needles: list = field(default_factory=list)                      # (seq, p, t_star, j_star)
    seed: int = 0

    def positions(self) -> np.ndarray:
        if self.q_pos is not None:
            return self.q_pos.astype(np.int64)
        return self.q_pos0 + np.arange(self.T, dtype=np.int64)

    def sequences(self) -> np.ndarray:
        if self.q_seq is not None:
            return self.q_seq.astype(np.int64)
        return np.zeros(self.T, dtype=np.int64)

    @property
    def n_blocks(self) -> int:
        return self.s_max // self.B


def make_workload(name: str, *, n_seq: int = 1, seq_len, T: int, H: int, d: int, B: int, m: int,
                  k: int, q_dtype: str, k_dtype: str, pooled_dtype: Optional[str] = None,
                  mode: str = "prefill", n_needles: int = 0, seed: int = BASE_SEED,
                  s_max: Optional[int] = None) -> Workload:
    """Build one seeded workload.

    mode = "prefill": one sequence, T queries at positions seq_len-T .. seq_len-1 (T == seq_len is a
                      full causal prefill; T < seq_len is a chunk against a longer prefix).
    mode = "decode" : n_seq sequences, one query each at its sequence's last position (T == n_seq).
    mode = "varlen" : n_seq sequences prefilled whole and packed one after the other
                      (T == sum(seq_len); q_seq / q_pos give every query's sequence and position).
    seq_len: int, or a sequence of n_seq ints.
    """
    ss_q, ss_k, ss_misc = np.random.SeedSequence(seed).spawn(3)
    rng = np.random.default_rng(ss_misc)
    seq_len = np.atleast_1d(np.asarray(seq_len, dtype=np.int64))
    if seq_len.size == 1 and n_seq > 1:
        seq_len = np.repeat(seq_len, n_seq)
    assert seq_len.size == n_seq
    if s_max is None:
        s_max = int(-(-int(seq_len.max()) // B) * B)
    assert s_max % B == 0 and s_max >= seq_len.max()
    if pooled_dtype is None:
        pooled_dtype = F32 if k_dtype == F32 else BF16

    # queries and gates first (needles point at them)
    q_bits = _cast(_normal(ss_q, (T, H, d)), q_dtype)
    w = rng.random((T, H), dtype=np.float32)

    if mode == "prefill":
        assert n_seq == 1 and T <= seq_len[0]
        q_pos0 = int(seq_len[0]) - T
        q_seq = None
        q_pos = None
        pos = q_pos0 + np.arange(T, dtype=np.int64)
        seqs = np.zeros(T, dtype=np.int64)
    elif mode == "decode":
        assert T == n_seq
        q_pos0 = 0
        q_seq = np.arange(T, dtype=np.int32)
        q_pos = (seq_len - 1).astype(np.int32)
        pos = q_pos.astype(np.int64)
        seqs = q_seq.astype(np.int64)
    elif mode == "varlen":
        assert T == int(seq_len.sum())
        q_pos0 = 0
        q_seq = np.repeat(np.arange(n_seq, dtype=np.int32), seq_len)
        q_pos = np.concatenate([np.arange(int(n), dtype=np.int32) for n in seq_len])
        pos = q_pos.astype(np.int64)
        seqs = q_seq.astype(np.int64)
    else:
        raise ValueError(mode)

    # keys, one sequence at a time (bounded host memory at 32 x 128K)
    if k_dtype == FP8:
        keys = np.zeros((n_seq, s_max, d), dtype=np.uint8)
        k_scale = np.ones((n_seq, s_max), dtype=np.float32)
    else:
        keys = np.zeros((n_seq, s_max, d), dtype=np.float32 if k_dtype == F32 else np.uint16)
        k_scale = None

    # needle plan (positions drawn before the keys so the stream order is fixed)
    needles = []
    for _ in range(n_needles):
        n = int(rng.integers(0, n_seq))
        p = int(rng.integers(0, int(seq_len[n])))
        cand = np.nonzero((seqs == n) & (pos >= p))[0]
        t_star = int(cand[rng.integers(0, cand.size)])
        j_star = int(rng.integers(0, H))
        needles.append((n, p, t_star, j_star))

    ss_seq = ss_k.spawn(n_seq)
    for n in range(n_seq):
        Ln = int(seq_len[n])
        nb = -(-Ln // B)
        ss_c, ss_t = ss_seq[n].spawn(2)
        cent = _normal(ss_c, (nb, d))
        kf = _normal(ss_t, (Ln, d))
        kf *= np.float32(0.5)
        kf += np.repeat(cent, B, axis=0)[:Ln]
        for (nn, p, t_star, j_star) in needles:
            if nn == n:
                v = _as_f32(q_bits[t_star, j_star], q_dtype)
                kf[p] = np.float32(3.0 * np.sqrt(1.25 * d)) * v / np.linalg.norm(v)
        if k_dtype == FP8:
            codes, sc = _to_fp8(kf)
            keys[n, :Ln] = codes
            k_scale[n, :Ln] = sc
        else:
            keys[n, :Ln] = _cast(kf, k_dtype)
        del kf

    return Workload(name=name, n_seq=n_seq, s_max=s_max, T=T, H=H, d=d, B=B, m=m, k=k,
                    q_dtype=q_dtype, k_dtype=k_dtype, pooled_dtype=pooled_dtype, keys=keys,
                    k_scale=k_scale, seq_len=seq_len.astype(np.int32), q=q_bits, w=w, q_seq=q_seq,
                    q_pos=q_pos, q_pos0=q_pos0, needles=needles, seed=seed)


def pack(wl: Workload, name: Optional[str] = None) -> Workload:
    """The sequences of a "varlen" workload laid end to end in ONE key stream, without padding
    between them (Section 4.1: blocks of the packed stream may straddle two sequences).  Query t
    keeps its data; its position becomes start(sequence) + position and it carries that start as
    its first visible position.  Pure data movement: same stored bits, new coordinates."""
    assert wl.q_seq is not None and wl.q_pos is not None and wl.q_lo is None
    lens = wl.seq_len.astype(np.int64)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    total = int(lens.sum())
    s_max = int(-(-total // wl.B) * wl.B)
    keys = np.zeros((1, s_max) + wl.keys.shape[2:], dtype=wl.keys.dtype)
    k_scale = None if wl.k_scale is None else np.ones((1, s_max), dtype=np.float32)
    for n in range(wl.n_seq):
        keys[0, starts[n]:starts[n] + lens[n]] = wl.keys[n, :lens[n]]
        if k_scale is not None:
            k_scale[0, starts[n]:starts[n] + lens[n]] = wl.k_scale[n, :lens[n]]
    seqs = wl.q_seq.astype(np.int64)
    return Workload(name=name or wl.name + "_packed", n_seq=1, s_max=s_max, T=wl.T, H=wl.H, d=wl.d, B=wl.B,
                    m=wl.m, k=wl.k, q_dtype=wl.q_dtype, k_dtype=wl.k_dtype, pooled_dtype=wl.pooled_dtype,
                    keys=keys, k_scale=k_scale, seq_len=np.array([total], dtype=np.int32), q=wl.q, w=wl.w,
                    q_seq=None, q_pos=(starts[seqs] + wl.q_pos).astype(np.int32), q_pos0=0,
                    q_lo=starts[seqs].astype(np.int32), needles=[], seed=wl.seed)


# The five benchmark configurations (shapes: Section 5.1 of the paper for B, m, k; H and d are
# the indexer sizes the benchmark definition fixes).
def config(name: str) -> Workload:
    if name == "tiny_f32":
        return make_workload(name, seq_len=1024, T=1024, H=4, d=64, B=64, m=4, k=128,
                             q_dtype=F32, k_dtype=F32, seed=BASE_SEED + 1)
    if name == "prefill16k_bf16":
        return make_workload(name, seq_len=16384, T=16384, H=64, d=128, B=128, m=32, k=2048,
                             q_dtype=BF16, k_dtype=BF16, n_needles=16, seed=BASE_SEED + 2)
    if name == "prefill64k_bf16":
        return make_workload(name, seq_len=65536, T=65536, H=64, d=128, B=128, m=64, k=2048,
                             q_dtype=BF16, k_dtype=BF16, n_needles=16, seed=BASE_SEED + 3)
    if name == "prefill64k_fp8":
        return make_workload(name, seq_len=65536, T=65536, H=64, d=128, B=128, m=64, k=2048,
                             q_dtype=BF16, k_dtype=FP8, n_needles=16, seed=BASE_SEED + 3)
    if name == "decode32x128k_bf16":
        rng = np.random.default_rng(BASE_SEED + 4000)
        lens = rng.integers(98304, 131072 + 1, size=32)
        return make_workload(name, n_seq=32, seq_len=lens, T=32, H=64, d=128, B=128, m=64, k=2048,
                             q_dtype=BF16, k_dtype=BF16, mode="decode", seed=BASE_SEED + 4,
                             s_max=131072)
    if name == "chunk16k_1m_fp8":
        return make_workload(name, seq_len=1048576, T=16384, H=64, d=128, B=128, m=128, k=2048,
                             q_dtype=BF16, k_dtype=FP8, n_needles=64, seed=BASE_SEED + 5)
    if name == "paper1024x64k_bf16":   # Section 5.1 shape: 1024 queries at the end of a 64K context
        return make_workload(name, seq_len=65536, T=1024, H=64, d=128, B=128, m=64, k=2048,
                             q_dtype=BF16, k_dtype=BF16, seed=BASE_SEED + 6)
    raise KeyError(name)


CONFIG_NAMES = ["tiny_f32", "prefill16k_bf16", "prefill64k_bf16", "prefill64k_fp8",
                "decode32x128k_bf16", "chunk16k_1m_fp8"]
