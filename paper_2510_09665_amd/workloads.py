"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *describes and draws inputs*: KV geometries (model shapes named in
the evaluation, section 8.1), page contents, token ids, slot mappings and request
mixes.  It holds none of the path's work (no gather, scatter, hashing, pool or index
logic) and is the one module that both the CPU oracle's tests and the GPU path's
tests and benchmark use, so that the two sides see identical inputs.

All randomness is numpy's PCG64 seeded with 0x5EED0000 + config id.
"""
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 0x5EED0000


@dataclass(frozen=True)
class KVGeometry:
    """Shape and byte strides of an engine's paged KV memory plus the chunk length.

    One allocation per layer; inside it the run of D*e bytes of (plane p, block b,
    in-block token o, head h) starts at
    p*plane_stride + b*block_stride + o*token_stride + h*head_stride.
    """
    L: int
    P: int
    H: int
    D: int
    e: int
    BS: int
    NB: int
    CT: int = 256
    layout: str = "NHD"          # "NHD": [P][NB][BS][H][D]   "HND": [P][NB][H][BS][D]
    block_pad: int = 0           # extra bytes after every block (exercises padded strides)
    order: str = "PN"            # "PN": planes outermost, as above; "NP": blocks outermost,
                                 # [NB][P][...]: the K and V page of a block are neighbours
    plane_stride: int = field(init=False)
    block_stride: int = field(init=False)
    token_stride: int = field(init=False)
    head_stride: int = field(init=False)

    def __post_init__(self):
        run = self.D * self.e
        if self.layout == "NHD":
            head, token = run, self.H * run
        elif self.layout == "HND":
            token, head = run, self.BS * run
        else:
            raise ValueError(self.layout)
        page = self.BS * self.H * run + self.block_pad
        if self.order == "PN":
            plane, block = self.NB * page, page
        elif self.order == "NP":
            plane, block = page, self.P * page
        else:
            raise ValueError(self.order)
        object.__setattr__(self, "head_stride", head)
        object.__setattr__(self, "token_stride", token)
        object.__setattr__(self, "block_stride", block)
        object.__setattr__(self, "plane_stride", plane)

    @property
    def R(self):
        """bytes of one token's row in one layer and plane"""
        return self.H * self.D * self.e

    @property
    def page_bytes(self):
        """bytes from one page (a block's share of one plane) to the next, padding included"""
        return self.BS * self.R + self.block_pad

    @property
    def layer_bytes(self):
        return self.P * self.NB * self.page_bytes

    @property
    def chunk_bytes(self):
        return self.L * self.P * self.CT * self.R

    @property
    def n_slots(self):
        return self.NB * self.BS


@dataclass(frozen=True)
class BlockMajorKV:
    """An engine layout with every layer in ONE allocation and blocks outermost,
    [NB][L][P][BS][H][D]: all of a block's KV (every layer, K and V) is one contiguous
    extent of L*P*page bytes.  Expressed with the same four strides: layer l starts
    layer_offset(l) bytes into the allocation, planes are a page apart and blocks
    L*P pages.  Carries the attributes a geometry needs (L P H D e BS NB CT and strides)."""
    shape: KVGeometry

    def __getattr__(self, name):            # L, P, H, D, e, BS, NB, CT, R, chunk_bytes, n_slots, ...
        return getattr(object.__getattribute__(self, "shape"), name)

    @property
    def page_bytes(self):
        return self.shape.BS * self.shape.R

    @property
    def plane_stride(self):
        return self.page_bytes

    @property
    def block_stride(self):
        return self.shape.L * self.shape.P * self.page_bytes

    @property
    def token_stride(self):
        return self.shape.R

    @property
    def head_stride(self):
        return self.shape.D * self.shape.e

    @property
    def total_bytes(self):
        return self.shape.NB * self.block_stride

    def layer_offset(self, layer):
        return layer * self.shape.P * self.page_bytes


# The five benchmark configurations.  NB where the configuration leaves it open:
# large enough that the store blocks and the fresh retrieve blocks are disjoint.
CONFIGS = {
    "tiny":        dict(id=1, geom=dict(L=2, P=2, H=4, D=64, e=2, BS=16, NB=64), tokens=256),
    "llama3_8b":   dict(id=2, geom=dict(L=32, P=2, H=8, D=128, e=2, BS=16, NB=8192), tokens=4096),
    "llama3_70b":  dict(id=3, geom=dict(L=80, P=2, H=8, D=128, e=2, BS=16, NB=8192), tokens=32768),
    "batch_8b":    dict(id=4, geom=dict(L=32, P=2, H=8, D=128, e=2, BS=16, NB=16384), tokens=None),
    "mla_bf16":    dict(id=5, geom=dict(L=61, P=1, H=1, D=576, e=2, BS=64, NB=1024), tokens=8192),
    "mla_fp8":     dict(id=5, geom=dict(L=61, P=1, H=1, D=576, e=1, BS=64, NB=1024), tokens=8192),
}


def page_view(geom, layer):
    """A layer's bytes (numpy array or torch tensor) seen as [P][NB][page_bytes]."""
    if geom.order == "PN":
        return layer.reshape(geom.P, geom.NB, geom.page_bytes)
    v = layer.reshape(geom.NB, geom.P, geom.page_bytes)
    return v.transpose(1, 0) if hasattr(v, "is_contiguous") else v.transpose(1, 0, 2)


def pages_to_layer(geom, pages):
    """Inverse of page_view: [P][NB][page_bytes] (array or tensor) to the layer's flat bytes."""
    if geom.order == "NP":
        pages = pages.transpose(1, 0) if hasattr(pages, "is_contiguous") else pages.transpose(1, 0, 2)
    if hasattr(pages, "is_contiguous"):
        return pages.contiguous().view(-1)
    return np.ascontiguousarray(pages).reshape(-1)


def geometry(name, **overrides):
    kw = dict(CONFIGS[name]["geom"])
    kw.update(overrides)
    return KVGeometry(**kw)


def rng_for(name, stream=0):
    return np.random.Generator(np.random.PCG64([SEED_BASE + CONFIGS[name]["id"], stream]))


def bf16_uniform(rng, n, block=1 << 20):
    """n bf16 values uniform in [-1, 1): drawn in fp32, rounded to nearest even, as uint16.
    Worked through in blocks that stay in cache (the 10 GiB of configuration 3 are drawn
    on the host); the values do not depend on the block size."""
    out = np.empty(n, dtype=np.uint16)
    buf = np.empty(min(block, max(n, 1)), dtype=np.float32)
    for i in range(0, n, block):
        f = buf[:min(block, n - i)]
        rng.random(out=f, dtype=np.float32)
        f *= np.float32(2.0)
        f -= np.float32(1.0)
        u = f.view(np.uint32)
        u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        out[i:i + f.size] = u >> np.uint32(16)
    return out


_FP8_OK = np.array([b for b in range(256) if b not in (0x7F, 0xFF, 0x80)], dtype=np.uint8)


def fp8_bytes(rng, n):
    """n fp8-e4m3 payload bytes, uniform over every encoding that is not a NaN
    (0x7F / 0xFF in the OCP format, 0x80 in the fnuz format)."""
    return _FP8_OK[rng.integers(0, _FP8_OK.size, n)]


def payload_bytes(rng, geom, nbytes):
    """nbytes of KV payload in geom's element type, as uint8."""
    if geom.e == 2:
        return bf16_uniform(rng, nbytes // 2).view(np.uint8)
    if geom.e == 1:
        return fp8_bytes(rng, nbytes)
    return rng.integers(0, 256, nbytes, dtype=np.uint8)


def sentinel_layer(geom, layer):
    """A full layer allocation of a repeating byte pattern that random payload will
    not reproduce over any run: used for 'every untouched byte is unchanged' checks."""
    pat = (np.arange(geom.layer_bytes, dtype=np.uint32) * np.uint32(2654435761) +
           np.uint32(layer * 97 + 13)) >> np.uint32(24)
    return pat.astype(np.uint8)


def random_layers(rng, geom):
    """All layers filled with payload (small geometries only)."""
    return [payload_bytes(rng, geom, geom.layer_bytes) for _ in range(geom.L)]


def tokens_for(rng, n, vocab=128256):
    return rng.integers(0, vocab, n, dtype=np.int64).astype(np.int32)


def pick_blocks(rng, geom, n_blocks, exclude=None):
    """n_blocks distinct block ids in seeded random order, avoiding `exclude`."""
    perm = rng.permutation(geom.NB)
    if exclude is not None:
        perm = perm[~np.isin(perm, np.asarray(exclude))]
    if perm.size < n_blocks:
        raise ValueError("pool of %d blocks cannot supply %d" % (geom.NB, n_blocks))
    return perm[:n_blocks].astype(np.int64)


def slots_from_blocks(geom, blocks, n_tokens):
    """Token t of the sequence lives in blocks[t // BS] at in-block offset t % BS."""
    t = np.arange(n_tokens, dtype=np.int64)
    return np.asarray(blocks, dtype=np.int64)[t // geom.BS] * geom.BS + t % geom.BS


def sequence(name, geom=None, stream=0, n_tokens=None):
    """One request of the named configuration: tokens, store slots, fresh retrieve slots."""
    geom = geom or geometry(name)
    rng = rng_for(name, stream)
    n = n_tokens if n_tokens is not None else CONFIGS[name]["tokens"]
    nb = -(-n // geom.BS)
    store_blocks = pick_blocks(rng, geom, nb)
    load_blocks = pick_blocks(rng, geom, nb, exclude=store_blocks)
    return dict(
        tokens=tokens_for(rng, n),
        store_blocks=store_blocks,
        load_blocks=load_blocks,
        store_slots=slots_from_blocks(geom, store_blocks, n),
        load_slots=slots_from_blocks(geom, load_blocks, n),
    )


def request_mix(name="batch_8b", geom=None, n_req=64, median=2048, sigma=1.0,
                lo=256, hi=16384, stream=0):
    """Batched multi-request retrieve: prefix lengths lognormal(median, sigma) clipped to
    [lo, hi] and rounded to whole chunks; each request hits a uniform-random leading
    fraction of its chunks; destination blocks are dealt from one global permutation so
    a request's pages are scattered among the other requests' pages."""
    geom = geom or geometry(name)
    rng = rng_for(name, stream)
    CT = geom.CT
    lens = np.clip(np.exp(np.log(median) + sigma * rng.standard_normal(n_req)), lo, hi)
    n_chunks = np.maximum(1, np.rint(lens / CT)).astype(np.int64)
    n_hit = np.rint(rng.random(n_req) * n_chunks).astype(np.int64)
    perm = rng.permutation(geom.NB).astype(np.int64)
    need = int((n_hit * (CT // geom.BS)).sum())
    if need > geom.NB:
        raise ValueError("request mix needs %d blocks, pool has %d" % (need, geom.NB))
    reqs, used = [], 0
    for r in range(n_req):
        toks = tokens_for(rng, int(n_chunks[r]) * CT)
        nb = int(n_hit[r]) * (CT // geom.BS)
        blocks = perm[used:used + nb]
        used += nb
        reqs.append(dict(tokens=toks, n_chunks=int(n_chunks[r]), n_hit=int(n_hit[r]),
                         load_blocks=blocks,
                         load_slots=slots_from_blocks(geom, blocks, int(n_hit[r]) * CT)))
    return reqs
