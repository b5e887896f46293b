"""Plumbing for the GPU parity tests: paged KV memory on the device beside a compact
host copy of the blocks a test touches, so the oracle can run on configurations whose
full page pool (16-40 GiB) should not be mirrored on the host.

Nothing here computes the path: the device side is filled and read back with torch
copies, the host side is handed to the oracle.
"""
import dataclasses

import numpy as np
import torch

from paper_2510_09665_amd import workloads as W


def sentinel_byte(layer):
    return (0x41 + 7 * layer) & 0xFF


class PagedKV:
    """Device pages of `geom` (every byte a per-layer sentinel) plus, for the listed
    blocks, payload that also lives in compact host layers: block blocks[i] of the
    device is block i of the compact geometry `gc`."""

    def __init__(self, geom, blocks, rng=None, device="cuda", fill="payload", threads=1):
        """threads > 1: the layers' payload is drawn in parallel, each layer from its own
        child generator of rng (for the configurations with GiBs of payload)."""
        self.g = geom
        self.blocks = np.asarray(blocks, dtype=np.int64)
        assert np.unique(self.blocks).size == self.blocks.size
        self.gc = dataclasses.replace(geom, NB=int(self.blocks.size))
        self._index = {int(b): i for i, b in enumerate(self.blocks)}
        self.dev = []
        self.host = []
        tb = torch.from_numpy(self.blocks).to(device)
        drawn = None
        if fill == "payload" and threads > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(threads) as ex:
                drawn = list(ex.map(lambda r: W.payload_bytes(r, geom, self.gc.layer_bytes), rng.spawn(geom.L)))
        for l in range(geom.L):
            d = torch.full((geom.layer_bytes,), sentinel_byte(l), dtype=torch.uint8, device=device)
            if fill == "payload":
                h = drawn[l] if drawn is not None else W.payload_bytes(rng, geom, self.gc.layer_bytes)
                W.page_view(geom, d)[:, tb] = W.page_view(self.gc, torch.from_numpy(h).to(device))
            else:
                h = np.full(self.gc.layer_bytes, sentinel_byte(l), dtype=np.uint8)
            self.dev.append(d)
            self.host.append(h)

    def compact_slots(self, slots):
        """The same tokens addressed in the compact geometry (negative slots kept)."""
        slots = np.asarray(slots, dtype=np.int64)
        out = slots.copy()
        ok = (slots >= 0) & (slots < self.g.n_slots)
        lut = np.full(self.g.NB, -1, dtype=np.int64)
        lut[self.blocks] = np.arange(self.blocks.size)
        cb = lut[slots[ok] // self.g.BS]
        assert (cb >= 0).all(), "slot outside the blocks this PagedKV tracks"
        out[ok] = cb * self.g.BS + slots[ok] % self.g.BS
        return out

    def device_blocks_to_host(self):
        """The tracked blocks as they are on the device now, in compact layout."""
        tb = torch.from_numpy(self.blocks).to(self.dev[0].device)
        g = self.g
        return [W.pages_to_layer(self.gc, W.page_view(g, d)[:, tb]).cpu().numpy() for d in self.dev]

    def untracked_blocks_untouched(self):
        """True if every block outside the tracked set still holds only the sentinel."""
        g = self.g
        keep = torch.ones(g.NB, dtype=torch.bool, device=self.dev[0].device)
        keep[torch.from_numpy(self.blocks).to(keep.device)] = False
        for l, d in enumerate(self.dev):
            v = W.page_view(g, d)[:, keep]
            if not bool((v == sentinel_byte(l)).all()):
                return False
        return True


def slots_to_device(slots, device="cuda"):
    return torch.from_numpy(np.ascontiguousarray(slots, dtype=np.int64)).to(device)


def assert_layers_equal(got, want, what=""):
    for l, (a, b) in enumerate(zip(got, want)):
        if not np.array_equal(a, b):
            bad = np.flatnonzero(a != b)
            raise AssertionError("%s layer %d: %d bytes differ, first at %d (got %d want %d)" %
                                 (what, l, bad.size, bad[0], a[bad[0]], b[bad[0]]))
