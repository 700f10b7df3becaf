"""Seeded synthetic inputs for the non-uniform all-to-all workloads.

This module only *makes inputs*: count matrices with the size distributions of
the paper's micro-benchmarks (uniform [0,S], normal, power-law, the degenerate
uniform all-to-all case; Section "Evaluation" and Section "Standard
distributions"), MPI_Alltoallv-style displacement arrays, and payload bytes.
It holds none of the all-to-all method's arithmetic and is shared by the CPU
oracle's tests and by the GPU path's tests and benchmark.

Everything is a pure function of a 64-bit seed through a counter-based
generator (splitmix64 of seed xor counter), so any part of an input can be
regenerated independently of any other part, on the host or on the device.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np

BASE_SEED = 0x241102581
_MASK64 = (1 << 64) - 1


# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------
def splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser applied element-wise to a uint64 array of counters."""
    with np.errstate(over="ignore"):
        z = (x.astype(np.uint64) + np.uint64(0x9E3779B97F4A7C15))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _hash_matrix(seed: int, P: int, stream: int = 0) -> np.ndarray:
    """u(i,j) = splitmix64(seed ^ stream-tag ^ (i*P + j)) as a P x P uint64 matrix."""
    ctr = np.arange(P * P, dtype=np.uint64)
    tag = np.uint64(((seed & _MASK64) ^ ((stream * 0xD1B54A32D192ED03) & _MASK64)) & _MASK64)
    return splitmix64(ctr ^ tag).reshape(P, P)


def _unit(u: np.ndarray) -> np.ndarray:
    """uint64 -> float64 in (0,1): top 53 bits, never exactly 0."""
    return ((u >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


# ----------------------------------------------------------------------------
# count matrices (bytes; row i = sender, column j = receiver)
# ----------------------------------------------------------------------------
def counts_uniform_elements(P: int, seed: int, max_elems: int, elem_bytes: int) -> np.ndarray:
    """count = elem_bytes * (u mod (max_elems+1)): uniform number of elements in [0, max_elems]."""
    u = _hash_matrix(seed, P)
    return ((u % np.uint64(max_elems + 1)).astype(np.int64) * elem_bytes).astype(np.int32)


def counts_uniform_bytes(P: int, seed: int, max_bytes: int) -> np.ndarray:
    """count = u mod (max_bytes+1): uniform byte counts in [0, max_bytes], any alignment."""
    u = _hash_matrix(seed, P)
    return (u % np.uint64(max_bytes + 1)).astype(np.int32)


def counts_zipf(P: int, seed: int, s: float = 1.2, max_bytes: int = 16384, quantum: int = 4) -> np.ndarray:
    """Power-law sizes: k in {1..max_bytes/quantum+1} with P(k) ~ k^-s by inverse CDF on the
    finite support; count = quantum*(k-1) bytes.  Many empty and tiny blocks, rare large ones."""
    kmax = max_bytes // quantum + 1
    k = np.arange(1, kmax + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    u = _unit(_hash_matrix(seed, P))
    idx = np.searchsorted(cdf, u, side="left")
    idx = np.minimum(idx, kmax - 1)
    return (idx.astype(np.int64) * quantum).astype(np.int32)


def counts_normal(P: int, seed: int, mean: float = 1024.0, sd: float = 256.0, quantum: int = 4) -> np.ndarray:
    """count = quantum*round(max(0, mean + sd*g)/quantum), g standard normal by Box-Muller from
    two hashed uniforms."""
    u1 = _unit(_hash_matrix(seed, P, stream=1))
    u2 = _unit(_hash_matrix(seed, P, stream=2))
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    v = np.maximum(0.0, mean + sd * g)
    return (np.rint(v / quantum).astype(np.int64) * quantum).astype(np.int32)


def counts_constant(P: int, nbytes: int) -> np.ndarray:
    """Every block has the same size: the uniform MPI_Alltoall special case."""
    return np.full((P, P), nbytes, dtype=np.int32)


def counts_fft_n1(P: int) -> np.ndarray:
    """The sparse FFT transpose pattern (Section "Fast Fourier transform", problem size N1): only
    ranks below ceil(0.625 P) hold data, and each of them fills its first ceil(0.78125 P) blocks
    with 8 FP64 values (64 bytes); every other block is empty."""
    workers = math.ceil(0.625 * P)
    filled = math.ceil(0.78125 * P)
    c = np.zeros((P, P), dtype=np.int32)
    c[:workers, :filled] = 8 * 8
    return c


def counts_fft_n2(P: int) -> np.ndarray:
    """The near-uniform FFT pattern (same section, problem size N2): every rank but the last sends
    64 FP64 values (512 bytes) per block, the last rank 16 FP64 values (128 bytes)."""
    c = np.full((P, P), 64 * 8, dtype=np.int32)
    c[P - 1, :] = 16 * 8
    return c


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Config:
    cfg: int
    P: int
    ranks_per_node: int          # 0 = flat
    radices: tuple               # flat: radix sweep; hierarchical single-radix call: radix sweep
    local_radix: Optional[int]   # set when the two radices are chosen separately
    global_radices: Optional[tuple]
    description: str

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg


CONFIGS = {
    1: Config(1, 16, 0, (2,), None, None,
              "P=16 flat r=2; counts 4*U{0..64} bytes; traceable int32 payload"),
    2: Config(2, 256, 0, (2, 4, 16, 256), None, None,
              "P=256 flat; counts U{0..1024} bytes, arbitrary alignment; random bytes"),
    3: Config(3, 1024, 16, (), 4, (2, 8, 64),
              "P=1024, 16 ranks/node x 64 nodes, r_l=4, r_g sweep; Zipf(1.2) <= 16 KiB, 4 B quantum"),
    4: Config(4, 4096, 0, (2, 8, 64, 4096), None, None,
              "P=4096 flat; counts normal(1 KiB, 256 B) clipped at 0, 4 B quantum; ~16 GiB"),
    5: Config(5, 2048, 32, (2, 16, 2048), None, None,
              "P=2048, 32 ranks/node x 64 nodes; all counts 256 B (uniform all-to-all)"),
}


def make_counts(cfg: int, P: Optional[int] = None) -> np.ndarray:
    """Count matrix of configuration `cfg`; `P` overrides the rank count (same distribution,
    same seed) for reduced-size parity cases."""
    c = CONFIGS[cfg]
    P = c.P if P is None else P
    if cfg == 1:
        return counts_uniform_elements(P, c.seed, 64, 4)
    if cfg == 2:
        return counts_uniform_bytes(P, c.seed, 1024)
    if cfg == 3:
        return counts_zipf(P, c.seed, 1.2, 16384, 4)
    if cfg == 4:
        return counts_normal(P, c.seed, 1024.0, 256.0, 4)
    if cfg == 5:
        return counts_constant(P, 256)
    raise KeyError(cfg)


# ----------------------------------------------------------------------------
# MPI_Alltoallv-style layouts
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Layout:
    """Displacements (bytes, int64) of an alltoallv problem over one send and one receive
    allocation that hold all P virtual ranks' buffers."""
    P: int
    sendcounts: np.ndarray   # [P,P] int32, [i,j] = bytes i sends to j
    sdispls: np.ndarray      # [P,P] int64, offset of block (i->j) in the send allocation
    recvcounts: np.ndarray   # [P,P] int32, [j,i] = bytes j receives from i
    rdispls: np.ndarray      # [P,P] int64, offset of block (i->j) in the receive allocation, at [j,i]
    send_bytes: int          # size of the send allocation
    recv_bytes: int          # size of the receive allocation

    @property
    def payload_bytes(self) -> int:
        return int(self.sendcounts.astype(np.int64).sum())


def _place(counts: np.ndarray, gap: int, permute_seed: Optional[int], align: int) -> tuple:
    """Lay the P*P blocks of `counts` (row-major: owner rank, then peer) into one allocation.
    gap: bytes left unused after every block; permute_seed: shuffle the order of the per-rank
    regions; align: round every block start up to this many bytes."""
    P = counts.shape[0]
    c = counts.astype(np.int64)
    step = c + gap
    if align > 1:
        step = (step + align - 1) // align * align
    row_bytes = step.sum(axis=1)
    order = np.arange(P)
    if permute_seed is not None:
        key = splitmix64(np.arange(P, dtype=np.uint64) ^ np.uint64(permute_seed & _MASK64))
        order = np.argsort(key, kind="stable")
    row_base = np.zeros(P, dtype=np.int64)
    acc = gap  # leading canary
    if align > 1:
        acc = (acc + align - 1) // align * align
    for r in order:
        row_base[r] = acc
        acc += int(row_bytes[r])
    within = np.cumsum(step, axis=1) - step
    displs = row_base[:, None] + within
    return displs.astype(np.int64), int(acc + gap)


def make_layout(sendcounts: np.ndarray, gap: int = 0, permute_seed: Optional[int] = None,
                align: int = 1) -> Layout:
    """Dense layout by default: per-rank send regions concatenated in rank order with blocks in
    destination order, receive regions likewise in source order.  `gap`/`permute_seed` give the
    canary-gap and permuted-region test variants."""
    P = sendcounts.shape[0]
    sendcounts = np.ascontiguousarray(sendcounts, dtype=np.int32)
    recvcounts = np.ascontiguousarray(sendcounts.T)
    sdispls, sbytes = _place(sendcounts, gap, permute_seed, align)
    rdispls, rbytes = _place(recvcounts, gap,
                             None if permute_seed is None else permute_seed + 1, align)
    return Layout(P, sendcounts, sdispls, recvcounts, rdispls, max(sbytes, 1), max(rbytes, 1))


# ----------------------------------------------------------------------------
# payloads
# ----------------------------------------------------------------------------
def payload_position_hash(seed: int, nbytes: int, start: int = 0) -> np.ndarray:
    """Send-allocation bytes [start, start+nbytes) of the position-hashed payload: the 8 bytes at
    offsets 8q..8q+7 are the little-endian bytes of splitmix64(seed ^ q).  Every 8-byte word is
    (almost surely) unique, so a block copied from the wrong place cannot compare equal."""
    q0 = start // 8
    q1 = (start + nbytes + 7) // 8
    words = splitmix64(np.arange(q0, q1, dtype=np.uint64) ^ np.uint64(seed & _MASK64))
    b = words.view(np.uint8)
    off = start - q0 * 8
    return b[off:off + nbytes].copy()


def payload_position_hash_torch(seed: int, nbytes: int, device, chunk_words: int = 1 << 25):
    """Same bytes as payload_position_hash(seed, nbytes, 0), produced with torch integer ops on
    `device` (in chunks), for buffers too large to make on the host and upload."""
    import torch

    nwords = (nbytes + 7) // 8
    out = torch.empty(nwords, dtype=torch.int64, device=device)

    def _c(v):  # python int -> signed 64-bit constant
        v &= _MASK64
        return v - (1 << 64) if v >= (1 << 63) else v

    def _lsr(t, k):  # logical shift right on int64
        return (t >> k) & ((1 << (64 - k)) - 1)

    for q0 in range(0, nwords, chunk_words):
        n = min(chunk_words, nwords - q0)
        z = torch.arange(q0, q0 + n, dtype=torch.int64, device=device)
        z = z ^ _c(seed)
        z = z + _c(0x9E3779B97F4A7C15)
        z = (z ^ _lsr(z, 30)) * _c(0xBF58476D1CE4E5B9)
        z = (z ^ _lsr(z, 27)) * _c(0x94D049BB133111EB)
        z = z ^ _lsr(z, 31)
        out[q0:q0 + n] = z
    return out.view(torch.uint8)[:nbytes]


def payload_position_hash_words32_torch(seed: int, word_index):
    """The 32-bit little-endian words of the position-hashed payload at the given 4-byte word
    indices (a torch int64 tensor on any device): word w is half (w & 1) of the 8-byte word
    splitmix64(seed ^ (w >> 1)).  Returned as int64 values in [0, 2^32)."""
    def _c(v):
        v &= _MASK64
        return v - (1 << 64) if v >= (1 << 63) else v

    def _lsr(t, k):
        return (t >> k) & ((1 << (64 - k)) - 1)

    z = (word_index >> 1) ^ _c(seed)
    z = z + _c(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _c(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _c(0x94D049BB133111EB)
    z = z ^ _lsr(z, 31)
    return (z >> ((word_index & 1) * 32)) & 0xFFFFFFFF


def payload_traceable_int32(layout: Layout) -> np.ndarray:
    """Configuration-1 payload: int32 element k of block (i->j) is (i<<20)|(j<<10)|k, so any
    received element names its origin.  Needs P <= 1024 and blocks of < 1024 int32 elements that
    start on 4-byte boundaries.  Bytes outside the blocks are 0xEE."""
    P = layout.P
    assert P <= 1024
    buf = np.full(layout.send_bytes, 0xEE, dtype=np.uint8)
    for i in range(P):
        for j in range(P):
            n = int(layout.sendcounts[i, j])
            assert n % 4 == 0 and n // 4 < 1024
            k = np.arange(n // 4, dtype=np.int64)
            v = ((i << 20) | (j << 10) | k).astype("<i4")
            o = int(layout.sdispls[i, j])
            buf[o:o + n] = v.view(np.uint8)
    return buf


def float32_bit_patterns(nbytes: int, seed: int) -> np.ndarray:
    """float32-typed payload that is moved bitwise: position-hashed words, with NaN, infinity,
    denormal and negative-zero bit patterns planted at regular positions."""
    b = payload_position_hash(seed, nbytes)
    n4 = nbytes // 4
    w = b[:n4 * 4].view("<u4")
    special = np.array([0x7FC00001, 0xFFC12345, 0x7F800000, 0xFF800000,
                        0x00000001, 0x807FFFFF, 0x80000000, 0x7FA00000], dtype="<u4")
    idx = np.arange(0, n4, 61)
    w[idx] = special[np.arange(idx.size) % special.size]
    return b
