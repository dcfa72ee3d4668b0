"""Host-side pools for tests: numpy arrays filled from the seeded generators, and
the closed-form index arithmetic the pins compare against.  No copy loop lives
here: expected values are always gathered through index arrays computed from
the layout formulas."""
import collections

import numpy as np

from paper_2510_02758_amd import workloads as W

CANARY = 0xA5

_ELEM = {"f16": 2, "bf16": 2, "fp8_e4m3": 1}
Sizes = collections.namedtuple("Sizes", "chunk block_bytes scale_chunk block_scale_bytes S")


def sizes(geom):
    """The sizes the interface header defines, worked out here from L, H, D, B and the element size alone, so that
    the pins' closed forms do not lean on the module that also feeds the library its shapes."""
    e = _ELEM[geom.dtype]
    chunk = geom.B * geom.H * geom.D * e                 # K or V of one block in one layer
    block_bytes = 2 * geom.L * chunk
    scale_chunk = geom.H * 4 if geom.scales else 0       # one fp32 per head
    block_scale_bytes = 2 * geom.L * scale_chunk
    return Sizes(chunk, block_bytes, scale_chunk, block_scale_bytes, block_bytes + block_scale_bytes)


def strides_for(geom, layout):
    """(data strides, scale strides, pool bytes, scale bytes) for a named layout."""
    if layout == "layer":
        return geom.strides, geom.scale_strides, geom.pool_bytes, geom.scale_bytes
    if layout == "block":
        sc = geom.scale_chunk
        return (geom.strides_block_major, (2 * sc, sc, 2 * geom.L * sc), geom.pool_bytes, geom.scale_bytes)
    if layout == "padded":
        bs = geom.chunk + 48
        ks = geom.N * bs + 32
        ls = 2 * ks + 64
        sbs = geom.scale_chunk + 8
        sks = geom.N * sbs + 4
        sls = 2 * sks + 12
        return (ls, ks, bs), (sls, sks, sbs), geom.L * ls, -(-geom.L * sls // 8) * 8
    raise ValueError(layout)


class HostPool:
    def __init__(self, geom, seed, layout="layer", slots=None, fill=True):
        self.geom, self.seed, self.layout = geom, seed, layout
        self.strides, self.scale_strides, pbytes, sbytes = strides_for(geom, layout)
        self.pool = W.fill_buffer_np(seed, pbytes, geom.dtype) if fill else np.zeros(pbytes, np.uint8)
        self.scale = None
        if geom.scales:
            self.scale = W.fill_buffer_np(seed ^ 0x5CA1E, sbytes, "raw") if fill else np.zeros(sbytes, np.uint8)
        self.slots = geom.N if slots is None else slots
        # spare bytes after the last slot (less than a slot): they must stay canary too
        self.sz = sizes(geom)
        self.staging = np.full(self.slots * self.sz.S + min(40, self.sz.S // 2), CANARY, dtype=np.uint8)

    def oracle(self, lib=None):
        """The C oracle over these arrays; `lib` may name another build of it, or be a
        factory (HostPool -> object with the Oracle methods) to put something else under the pins."""
        if callable(lib):
            return lib(self)
        from oracle.kv_oracle import Oracle
        g = self.geom
        return Oracle(g.L, g.H, g.D, g.B, g.e, g.N, self.pool, self.strides, self.staging,
                      scale=self.scale, scale_strides=self.scale_strides if g.scales else None, lib=lib)

    # ---- closed forms -------------------------------------------------
    def data_index(self, phys):
        """Pool byte offsets of blocks `phys`, in staging order [j][l][c][byte]."""
        g = self.geom
        ls, ks, bs = self.strides
        p = np.asarray(phys, dtype=np.int64)
        idx = (p[:, None, None, None] * bs + np.arange(g.L, dtype=np.int64)[None, :, None, None] * ls
               + np.arange(2, dtype=np.int64)[None, None, :, None] * ks
               + np.arange(self.sz.chunk, dtype=np.int64)[None, None, None, :])
        return idx.reshape(len(p), -1)

    def scale_index(self, phys):
        g = self.geom
        ls, ks, bs = self.scale_strides
        p = np.asarray(phys, dtype=np.int64)
        idx = (p[:, None, None, None] * bs + np.arange(g.L, dtype=np.int64)[None, :, None, None] * ls
               + np.arange(2, dtype=np.int64)[None, None, :, None] * ks
               + np.arange(self.sz.scale_chunk, dtype=np.int64)[None, None, None, :])
        return idx.reshape(len(p), -1)

    def block_image(self, phys, pool=None, scale=None):
        """What the staging slots of blocks `phys` must hold: array [len(phys), S]."""
        pool = self.pool if pool is None else pool
        out = pool[self.data_index(phys)]
        if self.geom.scales:
            scale = self.scale if scale is None else scale
            out = np.concatenate([out, scale[self.scale_index(phys)]], axis=1)
        return out

    def slots_view(self, staging=None):
        s = self.staging if staging is None else staging
        return s[: self.slots * self.sz.S].reshape(self.slots, self.sz.S)
