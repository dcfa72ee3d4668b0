"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only *produces inputs*: KV geometries, request lengths, block
tables and pool contents.  It contains nothing of the swap itself (no copy, no
placement of extents, no address of anything inside the staging arena),
imports neither the GPU binding nor the CPU oracle, and is the one piece both
sides are fed from.  `Geometry` does carry the sizes the interface defines for
a shape (bytes of a chunk, of a block, of a staging slot, the default strides):
callers need them to allocate pools and arenas.  The library and the oracle
each work these sizes out again from L, H, D, B and the element size, and so do
the tests' closed forms (tests/hostpool.py), so nothing is checked against
figures taken from here.

Pool contents are "address coded": the 64-bit word at byte offset 8*w of a
buffer is splitmix64(seed, w), a counter-based generator, so any part of a pool
far larger than host memory can be regenerated anywhere (numpy on the host,
torch integer ops on the device) from its offset alone.  Elements whose bit
pattern would be a NaN of the KV dtype are folded onto a finite pattern, since
serving systems never store NaNs in a KV cache; the swap itself is a byte copy
and never interprets the values.
"""
import dataclasses
from dataclasses import dataclass, field

import numpy as np

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

ELEM_BYTES = {"f16": 2, "bf16": 2, "fp8_e4m3": 1}
DTYPE_CODE = {"f16": 0, "bf16": 1, "fp8_e4m3": 2}


@dataclass(frozen=True)
class Geometry:
    """Shape of a paged KV pool.  Default strides are layer-major [L][2][N][chunk]."""
    L: int
    H: int
    D: int
    B: int
    dtype: str
    N: int
    scales: bool = False

    @property
    def e(self):
        return ELEM_BYTES[self.dtype]

    @property
    def chunk(self):
        return self.B * self.H * self.D * self.e

    @property
    def block_bytes(self):
        return 2 * self.L * self.chunk

    @property
    def scale_chunk(self):
        return self.H * 4 if self.scales else 0

    @property
    def block_scale_bytes(self):
        return 2 * self.L * self.scale_chunk

    @property
    def S(self):
        return self.block_bytes + self.block_scale_bytes

    @property
    def strides(self):
        """(layer_stride, kv_stride, block_stride) in bytes, layer-major."""
        return (2 * self.N * self.chunk, self.N * self.chunk, self.chunk)

    @property
    def strides_block_major(self):
        """[N][L][2][chunk]: a block is one contiguous run."""
        return (2 * self.chunk, self.chunk, self.block_bytes)

    @property
    def scale_strides(self):
        return (2 * self.N * self.scale_chunk, self.N * self.scale_chunk, self.scale_chunk)

    @property
    def pool_bytes(self):
        return self.N * self.block_bytes

    @property
    def scale_bytes(self):
        return self.N * self.block_scale_bytes


@dataclass(frozen=True)
class Workload:
    name: str
    geom: Geometry
    seed: int
    n_requests: int
    length_dist: tuple  # ("uniform", lo, hi) or ("lognormal", median, sigma, lo, hi)
    n_preempt: int      # requests swapped out (and back in)
    notes: str = ""


# The five benchmark configurations: KV shapes of Llama-3-8B / -70B class
# models and burst sizes in the range of the paper's controlled setups
# (Section 7.3, Table 2: bursts of 60-400 requests, inputs 512/1024 tokens,
# outputs 1024-4096 tokens).
def config(i, num_blocks=None, variant=0):
    """Configuration i.  variant 0 is the configuration's own seed; variants 1, 2, ... are further seeds
    of the same recipe (other lengths, other tables, other fill), for run-to-run spread."""
    wl = _config(i, num_blocks)
    if variant:
        wl = dataclasses.replace(wl, seed=wl.seed + (int(variant) << 8), name=wl.name + "/seed+%d" % variant)
    return wl


def _config(i, num_blocks):
    if i == 1:
        g = Geometry(2, 4, 64, 16, "f16", num_blocks or 1024)
        return Workload("tiny-fp16", g, 0x5EED0001, 8, ("uniform", 16, 256), 3)
    if i == 2:
        g = Geometry(32, 8, 128, 16, "bf16", num_blocks or 40000)
        return Workload("llama3-8b-burst64", g, 0x5EED0002, 64, ("uniform", 512, 4096), 64)
    if i == 3:
        g = Geometry(32, 8, 128, 16, "bf16", num_blocks or 40000)
        return Workload("llama3-8b-writethrough", g, 0x5EED0003, 256,
                        ("lognormal", 1024, 0.8, 16, 8128), 32)
    if i == 4:
        g = Geometry(80, 8, 128, 16, "bf16", num_blocks or (200 * 10**9) // (5 << 20))
        return Workload("llama3-70b-fragmented", g, 0x5EED0004, 128, ("uniform", 1024, 16384), 128)
    if i == 5:
        g = Geometry(32, 32, 128, 32, "fp8_e4m3", num_blocks or 16384, scales=True)
        return Workload("fp8-scales-mha", g, 0x5EED0005, 512, ("uniform", 256, 8192), 512)
    raise ValueError(i)


# ------------------------------------------------------------------ lengths

def request_lengths(seed, n, dist):
    """Token counts of n requests, int32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if dist[0] == "uniform":
        _, lo, hi = dist
        return rng.integers(lo, hi + 1, size=n).astype(np.int32)
    if dist[0] == "lognormal":
        _, median, sigma, lo, hi = dist
        x = np.exp(np.log(median) + sigma * rng.standard_normal(n))
        return np.clip(np.rint(x), lo, hi).astype(np.int32)
    raise ValueError(dist)


def blocks_for(lengths, B):
    lengths = np.asarray(lengths, dtype=np.int64)
    return ((lengths + B - 1) // B).astype(np.int64)


# ------------------------------------------------------------- block tables

def block_tables(seed, N, n_blocks_per_req):
    """Random block tables: prefix slices of one seeded permutation of [0, N).

    Returns (offsets int32[n+1], block_ids int32[total], free int32[N-total]);
    `free` is the rest of the permutation, i.e. a shuffled free list.
    """
    nb = np.asarray(n_blocks_per_req, dtype=np.int64)
    total = int(nb.sum())
    if total > N:
        raise ValueError("requests need %d blocks, pool has %d" % (total, N))
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xB10C))
    perm = rng.permutation(N).astype(np.int32)
    offsets = np.zeros(len(nb) + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(nb)
    return offsets, perm[:total].copy(), perm[total:].copy()


def fragmented_tables(seed, N, n_blocks_per_req, free_fraction=0.5):
    """Tables drawn from a pool in which a random `free_fraction` of the blocks was freed.

    The remaining blocks stay owned by foreign requests (they act as canaries
    between the blocks handed out here).  Returns (offsets, block_ids, free).
    """
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xF4A6))
    freed = np.flatnonzero(rng.random(N) < free_fraction).astype(np.int32)
    rng.shuffle(freed)
    nb = np.asarray(n_blocks_per_req, dtype=np.int64)
    total = int(nb.sum())
    if total > len(freed):
        raise ValueError("requests need %d blocks, only %d were freed" % (total, len(freed)))
    offsets = np.zeros(len(nb) + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(nb)
    return offsets, freed[:total].copy(), freed[total:].copy()


def pick(seed, n, k):
    """k distinct indices out of n, seeded, in random order."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x91C4))
    return rng.permutation(n)[:k]


def csr_take(offsets, ids, rows):
    """Sub-CSR holding the given rows, in the given order."""
    parts = [ids[offsets[r]:offsets[r + 1]] for r in rows]
    out_off = np.zeros(len(rows) + 1, dtype=np.int32)
    out_off[1:] = np.cumsum([len(p) for p in parts])
    out_ids = np.concatenate(parts).astype(np.int32) if parts else np.zeros(0, np.int32)
    return out_off, out_ids


# --------------------------------------------------------------- pool fill

def _mix_np(seed, w):
    """splitmix64 output for counter values w (uint64 array)."""
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & _M64) + (w + np.uint64(1)) * np.uint64(_GOLD))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_C1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_C2)
        z = z ^ (z >> np.uint64(31))
    return z


def _fold_nan_np(raw, dtype):
    """raw: uint8 array (length multiple of the element size), folded in place."""
    if dtype == "bf16":
        x = raw.view(np.uint16)
        m = (x & 0x7F80) == 0x7F80
        x[m] &= np.uint16(0xFF7F)
    elif dtype == "f16":
        x = raw.view(np.uint16)
        m = (x & 0x7C00) == 0x7C00
        x[m] &= np.uint16(0xFBFF)
    elif dtype == "fp8_e4m3":
        m = (raw & 0x7F) == 0x7F
        raw[m] &= np.uint8(0xFE)
    elif dtype == "raw":
        pass
    else:
        raise ValueError(dtype)
    return raw


def fill_bytes_np(seed, byte_offset, nbytes, dtype):
    """Content of bytes [byte_offset, byte_offset+nbytes) of a buffer filled with `seed`.

    byte_offset and nbytes must be multiples of 8.
    """
    assert byte_offset % 8 == 0 and nbytes % 8 == 0
    w = np.arange(byte_offset // 8, (byte_offset + nbytes) // 8, dtype=np.uint64)
    raw = _mix_np(seed, w).view(np.uint8)
    return _fold_nan_np(raw, dtype)


def fill_buffer_np(seed, nbytes, dtype):
    """A whole buffer of nbytes as a uint8 array (a ragged last word is cut short)."""
    out = np.empty(nbytes, dtype=np.uint8)
    step = 1 << 26
    for o in range(0, nbytes, step):
        n = min(step, nbytes - o)
        out[o:o + n] = fill_bytes_np(seed, o, -(-n // 8) * 8, dtype)[:n]
    return out


def _s64(v):
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix_torch(seed, w):
    """The same generator on a torch int64 tensor (two's complement wrap-around)."""
    def lsr(z, k):
        return (z >> k) & ((1 << (64 - k)) - 1)
    z = (w + 1) * _s64(_GOLD) + _s64(seed)
    z = (z ^ lsr(z, 30)) * _s64(_C1)
    z = (z ^ lsr(z, 27)) * _s64(_C2)
    return z ^ lsr(z, 31)


def _fold_nan_torch(raw, dtype):
    import torch
    if dtype == "bf16":
        x = raw.view(torch.int16)
        x.copy_(torch.where((x & 0x7F80) == 0x7F80, x & ~0x0080, x))
    elif dtype == "f16":
        x = raw.view(torch.int16)
        x.copy_(torch.where((x & 0x7C00) == 0x7C00, x & ~0x0400, x))
    elif dtype == "fp8_e4m3":
        x = raw.view(torch.int8)
        x.copy_(torch.where((x & 0x7F) == 0x7F, x & ~0x01, x))
    elif dtype != "raw":
        raise ValueError(dtype)
    return raw


def fill_bytes_torch(seed, byte_offset, nbytes, dtype, device):
    """torch counterpart of fill_bytes_np -> uint8 tensor on `device`."""
    import torch
    assert byte_offset % 8 == 0 and nbytes % 8 == 0
    w = torch.arange(byte_offset // 8, (byte_offset + nbytes) // 8, dtype=torch.int64, device=device)
    raw = _mix_torch(seed, w).view(torch.uint8)
    return _fold_nan_torch(raw, dtype)


def fill_words_torch(seed, word_index, dtype):
    """Content of the 64-bit words `word_index` (int64 tensor, any shape) of a buffer filled
    with `seed` -> uint8 tensor of shape word_index.shape + (8,), on the same device."""
    raw = _mix_torch(seed, word_index.contiguous()).view(word_index.dtype)
    import torch
    out = raw.view(torch.uint8).view(*word_index.shape, 8)
    return _fold_nan_torch(out, dtype)


def fill_buffer_torch(seed, buf, dtype, piece=1 << 28):
    """Fill a uint8 tensor in place, `piece` bytes at a time.  Returns when the fill has finished: the swap
    library runs on streams of its own, which do not wait for the stream torch filled the buffer on."""
    import torch
    n = buf.numel()
    for o in range(0, n, piece):
        m = min(piece, n - o)
        buf[o:o + m] = fill_bytes_torch(seed, o, m, dtype, buf.device)
    if buf.is_cuda:
        torch.cuda.synchronize(buf.device)
    return buf
