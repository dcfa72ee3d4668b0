"""Device-side checks for pools too large to mirror on the host.

Pools are address coded (workloads.fill_*): the expected content of any chunk follows from
its byte offset, so a block that was moved can be checked on the GPU with torch integer ops:
block `holder` must now hold what block `origin` was filled with.  Nothing here calls the
library under test or the oracle.
"""
import numpy as np
import torch

from paper_2510_02758_amd import workloads as W


def _plane_rows(buf, plane_off, N, stride, width):
    """[N, width] strided view of one (layer, K|V) plane of a flat uint8 buffer."""
    return torch.as_strided(buf, (N, width), (stride, 1), storage_offset=plane_off)


def count_wrong_blocks(pool, geom, strides, seed, holder, origin, dtype=None, width=None, max_rows=4096):
    """Number of (plane, block) pairs where block holder[i] does not hold the fill of block
    origin[i].  Works plane by plane so temporaries stay small."""
    ls, ks, bs = strides
    width = geom.chunk if width is None else width
    dtype = geom.dtype if dtype is None else dtype
    assert width % 8 == 0 and bs % 8 == 0 and ls % 8 == 0 and ks % 8 == 0
    dev = pool.device
    holder = torch.as_tensor(np.asarray(holder, dtype=np.int64), device=dev)
    origin = torch.as_tensor(np.asarray(origin, dtype=np.int64), device=dev)
    col = torch.arange(width // 8, dtype=torch.int64, device=dev)
    wrong = 0
    for l in range(geom.L):
        for c in range(2):
            off = l * ls + c * ks
            rows = _plane_rows(pool, off, geom.N, bs, width)
            for a in range(0, len(holder), max_rows):
                h, o = holder[a:a + max_rows], origin[a:a + max_rows]
                words = (off + o * bs)[:, None] // 8 + col[None, :]
                want = W.fill_words_torch(seed, words, dtype).reshape(len(h), width)
                got = rows.index_select(0, h)
                wrong += int((got != want).any(dim=1).sum())
    return wrong


def changed_blocks(pool, geom, strides, seed, dtype=None, width=None, piece_rows=8192):
    """Sorted ids of blocks whose content differs from their own fill in ANY plane
    (i.e. every block something was written into)."""
    ls, ks, bs = strides
    width = geom.chunk if width is None else width
    dtype = geom.dtype if dtype is None else dtype
    dev = pool.device
    col = torch.arange(width // 8, dtype=torch.int64, device=dev)
    dirty = torch.zeros(geom.N, dtype=torch.bool, device=dev)
    for l in range(geom.L):
        for c in range(2):
            off = l * ls + c * ks
            rows = _plane_rows(pool, off, geom.N, bs, width)
            for a in range(0, geom.N, piece_rows):
                b = min(geom.N, a + piece_rows)
                ids = torch.arange(a, b, dtype=torch.int64, device=dev)
                words = (off + ids * bs)[:, None] // 8 + col[None, :]
                want = W.fill_words_torch(seed, words, dtype).reshape(b - a, width)
                dirty[a:b] |= (rows[a:b] != want).any(dim=1)
    return torch.nonzero(dirty).flatten().cpu().numpy()


def host_blocks(geom, strides, seed, phys, dtype=None, width=None):
    """numpy image [len(phys), 2L*width] of the ORIGINAL fill of blocks `phys`, in (l, c) order:
    the data part of a staging slot (or the scale part, with the scale strides/width/seed)."""
    ls, ks, bs = strides
    width = geom.chunk if width is None else width
    dtype = geom.dtype if dtype is None else dtype
    out = np.empty((len(phys), 2 * geom.L, width), dtype=np.uint8)
    for i, p in enumerate(np.asarray(phys, dtype=np.int64)):
        for l in range(geom.L):
            for c in range(2):
                out[i, 2 * l + c] = W.fill_bytes_np(seed, l * ls + c * ks + int(p) * bs, width, dtype)
    return out.reshape(len(phys), -1)


def compact_mirror(geom, strides, seed, phys, extra_blocks, scale_seed=None):
    """Host pool of len(phys)+extra_blocks blocks whose block i holds the original fill of
    block phys[i] (the sparse mirror the oracle runs on).  Returns (Geometry, pool, scale)."""
    n = len(phys)
    gc = W.Geometry(geom.L, geom.H, geom.D, geom.B, geom.dtype, n + extra_blocks, scales=geom.scales)
    pool = np.zeros(gc.pool_bytes, dtype=np.uint8)
    img = host_blocks(geom, strides, seed, phys).reshape(n, geom.L, 2, geom.chunk)
    pv = pool.reshape(gc.L, 2, gc.N, gc.chunk)
    pv[:, :, :n, :] = img.transpose(1, 2, 0, 3)
    scale = None
    if geom.scales:
        scale = np.zeros(gc.scale_bytes, dtype=np.uint8)
        simg = host_blocks(geom, geom.scale_strides, scale_seed, phys, dtype="raw", width=geom.scale_chunk)
        sv = scale.reshape(gc.L, 2, gc.N, gc.scale_chunk)
        sv[:, :, :n, :] = simg.reshape(n, geom.L, 2, geom.scale_chunk).transpose(1, 2, 0, 3)
    return gc, pool, scale
