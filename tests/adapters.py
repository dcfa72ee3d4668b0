"""Adapters that let the oracle's pins (test_oracle_pins.py) drive the GPU library.

Both expose the Oracle class's methods over a HostPool:
  PlanOnlyAdapter  library under KV_PLAN_ONLY (no GPU): bookkeeping and descriptor
                   lists come from the library; a numpy stub applies the
                   descriptors to the host arrays.  Tests the host logic on CPU.
  GpuAdapter       the real thing: the pool lives on the device, the arena is pinned
                   host memory; host arrays are synchronised around every call so the
                   pins' numpy checks see what the kernels did.
"""
import numpy as np

from paper_2510_02758_amd import kvswap as kv


class _Base:
    def __init__(self, hp):
        self.hp = hp

    def reserve(self, req_id, max_blocks):
        return self.kp.reserve(req_id, max_blocks)

    def release(self, req_id):
        return self.kp.release(req_id)

    def query(self, req_id):
        rc, q = self.kp.query(req_id)
        return rc, q

    def close(self):
        self.kp.close()


class PlanOnlyAdapter(_Base):
    def __init__(self, hp):
        super().__init__(hp)
        g = hp.geom
        self.kp = kv.KVPool(g, strides=hp.strides, scale_strides=hp.scale_strides if g.scales else None,
                            flags=kv.KV_PLAN_ONLY, staging_bytes=hp.slots * g.S)

    def _apply_out(self):
        phys, slot = self.kp.last_plan()
        if len(phys):
            self.hp.slots_view()[slot] = self.hp.block_image(phys)

    def swap_out(self, req_ids, offsets, block_ids, num_tokens):
        rc = self.kp.swap_out(req_ids, offsets, block_ids, num_tokens)
        if rc == kv.KV_OK:
            self._apply_out()
        return rc

    def swap_out_delta(self, req_ids, offsets, block_ids, num_tokens, budget=0, flags=0):
        rc, moved = self.kp.swap_out_delta(req_ids, offsets, block_ids, num_tokens, budget, flags)
        if rc == kv.KV_OK:
            self._apply_out()
        return rc, moved

    def swap_in(self, req_ids, offsets, new_block_ids, flags=0):
        rc = self.kp.swap_in(req_ids, offsets, new_block_ids, flags)
        if rc == kv.KV_OK:
            phys, slot = self.kp.last_plan()
            if len(phys):
                hp, g = self.hp, self.hp.geom
                img = hp.slots_view()[slot]
                hp.pool[hp.data_index(phys)] = img[:, :g.block_bytes]
                if g.scales:
                    hp.scale[hp.scale_index(phys)] = img[:, g.block_bytes:]
        return rc

    def move_blocks(self, src_ids, dst_ids):
        rc = self.kp.move_blocks(src_ids, dst_ids)
        if rc == kv.KV_OK:
            src, dst = self.kp.last_plan()
            if len(src):
                hp = self.hp
                hp.pool[hp.data_index(dst)] = hp.pool[hp.data_index(src)]
                if hp.geom.scales:
                    hp.scale[hp.scale_index(dst)] = hp.scale[hp.scale_index(src)]
        return rc


class GpuAdapter(_Base):
    """flags: kv.KV_PATH_ZEROCOPY / kv.KV_PATH_DMA / kv.KV_STAGING_DEVICE."""

    def __init__(self, hp, flags=0, bounce_slots=3, tune=()):
        import torch
        super().__init__(hp)
        g = hp.geom
        dev = torch.device("cuda:0")
        self.torch = torch
        self.dev_staging = bool(flags & kv.KV_STAGING_DEVICE)
        self.pool = torch.from_numpy(hp.pool).to(dev)
        self.scale = torch.from_numpy(hp.scale).to(dev) if g.scales else None
        if self.dev_staging:
            self.staging = torch.from_numpy(hp.staging).to(dev)
        else:
            self.staging = torch.from_numpy(hp.staging.copy()).pin_memory()
            hp.staging = self.staging.numpy()  # the pins now look at the pinned arena itself
        bounce = None
        if flags & kv.KV_PATH_DMA:
            bounce = torch.zeros(2 * bounce_slots * g.S, dtype=torch.uint8, device=dev)
        self.kp = kv.KVPool(g, self.pool, self.staging, scale=self.scale, bounce=bounce, strides=hp.strides,
                            scale_strides=hp.scale_strides if g.scales else None, flags=flags)
        for what, value in tune:
            assert self.kp.tune(what, value) == kv.KV_OK

    def _push(self):
        t = self.torch
        self.pool.copy_(t.from_numpy(self.hp.pool))
        if self.scale is not None:
            self.scale.copy_(t.from_numpy(self.hp.scale))
        if self.dev_staging:
            self.staging.copy_(t.from_numpy(self.hp.staging))
        t.cuda.synchronize()

    def _pull(self):
        assert self.kp.sync() == kv.KV_OK
        self.torch.cuda.synchronize()
        self.hp.pool[:] = self.pool.cpu().numpy()
        if self.scale is not None:
            self.hp.scale[:] = self.scale.cpu().numpy()
        if self.dev_staging:
            self.hp.staging[:] = self.staging.cpu().numpy()

    def swap_out(self, req_ids, offsets, block_ids, num_tokens):
        self._push()
        rc = self.kp.swap_out(req_ids, offsets, block_ids, num_tokens)
        self._pull()
        return rc

    def swap_out_delta(self, req_ids, offsets, block_ids, num_tokens, budget=0, flags=0):
        self._push()
        rc, moved = self.kp.swap_out_delta(req_ids, offsets, block_ids, num_tokens, budget, flags)
        self._pull()
        return rc, moved

    def swap_in(self, req_ids, offsets, new_block_ids, flags=0):
        self._push()
        rc = self.kp.swap_in(req_ids, offsets, new_block_ids, flags)
        self._pull()
        return rc

    def move_blocks(self, src_ids, dst_ids):
        self._push()
        rc = self.kp.move_blocks(src_ids, dst_ids)
        self._pull()
        return rc
