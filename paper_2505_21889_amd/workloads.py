"""Seeded synthetic serving batches for the EFIM extend-attention path.

This module only draws inputs: request lengths, block tables and random bf16
tensors.  It contains none of the method's arithmetic (no RoPE, no attention,
no cache addressing) so that both the HIP library's tests and the independent
CPU oracle can be fed from it.

The paper serves two 7B-class rotary decoder models (Sec. 4) to 16 closed-loop
users with prompts of about 2.1-2.4k tokens of which only the incremental part
is new (Sec. 2.2, Sec. 4.2).  Its prompts come from benchmark suites and an
online service that are not reproduced here; the batches below are synthetic
stand-ins with the same structure -- ragged cached/new lengths, paged cache
with shuffled physical pages, Gaussian activations.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

POISON_BITS = 0xFFFF  # a NaN bit pattern in bf16: marks bytes that must never matter


@dataclass
class WorkloadSpec:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    rope_base: float
    sigma: float
    seed: int
    describe: str


SPECS = {
    "c1": WorkloadSpec("c1", 1, 4, 4, 64, 16, 1.0e4, 1.0, 1000,
                       "tiny extend: 1 request, 4/4 heads, d64, cached 256, inc 32"),
    "c2": WorkloadSpec("c2", 16, 32, 32, 128, 16, 1.0e4, 1.0, 1001,
                       "7B-shaped MHA: 16 requests, 32/32 heads, d128, cached U[1024,4096], inc U[16,128]"),
    "c3": WorkloadSpec("c3", 32, 28, 4, 128, 16, 1.0e6, 1.0, 1002,
                       "GQA 28/4: 32 requests, d128, cached U[2048,8192], inc U[8,64]"),
    "c4": WorkloadSpec("c4", 4, 32, 8, 128, 16, 1.0e6, 0.5, 1003,
                       "long-context infilling: 4 requests, 32/8 heads, d128, cached 16384, inc 512"),
    "c5": WorkloadSpec("c5", 64, 32, 8, 128, 16, 1.0e6, 1.0, 1004,
                       "mixed serving step: 64 requests, 32/8 heads, d128; half hits "
                       "(cached U[512,8192], inc U[1,256]), half misses (cached 0, new U[1024,4096])"),
    # one round of the multi-user infilling service of EFIM Sec. 4.2 (lengths come from
    # replay_documents and a session pool, never from draw_lengths); the two head layouts are
    # those of the two models the paper serves
    "replay": WorkloadSpec("replay", 16, 32, 8, 128, 16, 5.0e5, 1.0, 1005,
                           "service replay, GQA 32/8, d128: 16 users x 5 rounds, prompts of ~2355 tokens"),
    "replay_mha": WorkloadSpec("replay_mha", 16, 32, 32, 128, 16, 1.0e5, 1.0, 1006,
                               "service replay, MHA 32/32, d128: 16 users x 5 rounds, prompts of ~2355 tokens"),
}

REPLAY_USERS = 16
REPLAY_ROUNDS = 5
REPLAY_VOCAB = 32000            # content token ids are drawn below this; markers sit above it
REPLAY_MARKERS = (32001, 32002, 32003)


def replay_documents(seed=1005, users=REPLAY_USERS, rounds=REPLAY_ROUNDS):
    """Token sequences of the closed-loop service of EFIM Sec. 4.2: ``rounds`` lists of
    ``users`` (prefix, suffix) pairs.  Every user starts from a document split at the
    insertion point (prefix and suffix each U[600,1480] tokens) and in every later round has
    typed U[16,256] more tokens at the tail of the prefix; the suffix never changes.  With the
    three markers the prompts average 2355 tokens over the five rounds, the paper's figure."""
    rng = np.random.default_rng(seed)
    docs = []
    for _ in range(users):
        prefix = rng.integers(0, REPLAY_VOCAB, int(rng.integers(600, 1481))).astype(np.int32)
        suffix = rng.integers(0, REPLAY_VOCAB, int(rng.integers(600, 1481))).astype(np.int32)
        docs.append((prefix, suffix))
    out = [list(docs)]
    for _ in range(1, rounds):
        nxt = []
        for prefix, suffix in out[-1]:
            typed = rng.integers(0, REPLAY_VOCAB, int(rng.integers(16, 257))).astype(np.int32)
            nxt.append((np.concatenate([prefix, typed]), suffix))
        out.append(nxt)
    return out


def draw_lengths(name, rng):
    """(cached_len, new_len) int32 arrays for a named workload; bounds inclusive."""
    s = SPECS[name]
    b = s.batch
    if name == "c1":
        c, n = np.full(b, 256), np.full(b, 32)
    elif name == "c2":
        c, n = rng.integers(1024, 4097, b), rng.integers(16, 129, b)
    elif name == "c3":
        c, n = rng.integers(2048, 8193, b), rng.integers(8, 65, b)
    elif name == "c4":
        c, n = np.full(b, 16384), np.full(b, 512)
    elif name == "c5":
        hit = np.zeros(b, dtype=bool)
        hit[rng.permutation(b)[: b // 2]] = True
        c = np.where(hit, rng.integers(512, 8193, b), 0)
        n = np.where(hit, rng.integers(1, 257, b), rng.integers(1024, 4097, b))
    else:
        raise KeyError(name)
    return c.astype(np.int32), n.astype(np.int32)


def gaussian_bf16(rng, shape, sigma):
    """bf16 bit patterns (uint16) of N(0, sigma) samples, rounded by torch's cast."""
    x = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(sigma)
    t = torch.from_numpy(x).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


@dataclass
class ExtendBatch:
    """One serving step's inputs.  bf16 tensors are uint16 bit patterns."""
    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    rope_base: float
    sigma: float
    cached_len: np.ndarray            # int32[B]
    new_len: np.ndarray               # int32[B]
    block_table: np.ndarray           # int32[B, max_pages_per_req]
    num_pages: int                    # pages in each cache array (used + spare)
    q_new: np.ndarray                 # uint16[T, Hq, D]  raw new queries
    k_new: np.ndarray                 # uint16[T, Hkv, D] raw new keys
    v_new: np.ndarray                 # uint16[T, Hkv, D] new values
    k_hist: np.ndarray | None = None  # uint16[sum(C), Hkv, D] raw keys of the cached tokens
    v_hist: np.ndarray | None = None  # uint16[sum(C), Hkv, D] values of the cached tokens
    extra: dict = field(default_factory=dict)

    @property
    def batch(self):
        return int(self.cached_len.shape[0])

    @property
    def total_new(self):
        return int(self.new_len.sum())

    @property
    def max_pages_per_req(self):
        return int(self.block_table.shape[1])

    def cache_shape(self):
        return (self.num_pages, self.num_kv_heads, self.page_size, self.head_dim)


def make_block_table(cached_len, new_len, page_size, rng, spare_fraction=0.125):
    """Disjoint shuffled physical pages for every request.

    Entries past a request's last page point at one of the spare pages, which
    callers keep filled with POISON_BITS: a stray read shows up as NaN instead
    of an illegal address.
    Returns (block_table int32[B, max_pages], num_pages).
    """
    need = [-(-(int(c) + int(n)) // page_size) for c, n in zip(cached_len, new_len)]
    used = int(sum(need))
    spare = max(2, int(np.ceil(used * spare_fraction)))
    num_pages = used + spare
    perm = rng.permutation(num_pages).astype(np.int32)
    max_pages = max(need) if need else 0
    max_pages = max(1, max_pages)
    table = np.empty((len(need), max_pages), dtype=np.int32)
    spare_ids = perm[used:]
    at = 0
    for r, k in enumerate(need):
        table[r, :k] = perm[at:at + k]
        table[r, k:] = spare_ids[r % len(spare_ids)]
        at += k
    return table, num_pages


def make_batch(name, seed=None, with_history=True, lengths=None, heads=None,
               head_dim=None, page_size=None, sigma=None, rope_base=None, with_tensors=True):
    """Draw a batch of the named workload.

    ``lengths=(cached_len, new_len)`` overrides the drawn lengths (used by the
    sweeps that fix the incremental length); the other keyword arguments
    override single fields of the spec.  With ``with_history`` the raw keys and
    values of the cached tokens are drawn too, so that a cache can be built by
    appending them at positions 0..C-1.
    """
    s = SPECS[name]
    rng = np.random.default_rng(s.seed if seed is None else seed)
    hq, hkv = heads if heads is not None else (s.num_q_heads, s.num_kv_heads)
    d = head_dim or s.head_dim
    p = page_size or s.page_size
    sg = s.sigma if sigma is None else sigma
    base = s.rope_base if rope_base is None else rope_base
    if lengths is None:
        c, n = draw_lengths(name, rng)
    else:
        c = np.asarray(lengths[0], dtype=np.int32)
        n = np.asarray(lengths[1], dtype=np.int32)
    table, num_pages = make_block_table(c, n, p, rng)
    t = int(n.sum())
    if not with_tensors:
        # lengths and block table only: callers draw the tensors themselves (on the device)
        return ExtendBatch(name, hq, hkv, d, p, base, sg, c, n, table, num_pages, None, None, None)
    q = gaussian_bf16(rng, (t, hq, d), sg)
    k = gaussian_bf16(rng, (t, hkv, d), sg)
    v = gaussian_bf16(rng, (t, hkv, d), sg)
    kh = vh = None
    if with_history:
        tc = int(c.sum())
        kh = gaussian_bf16(rng, (tc, hkv, d), sg)
        vh = gaussian_bf16(rng, (tc, hkv, d), sg)
    return ExtendBatch(name, hq, hkv, d, p, base, sg, c, n, table, num_pages, q, k, v, kh, vh)


def poisoned_cache(batch):
    """A cache array of the batch's shape with every element set to POISON_BITS."""
    return np.full(batch.cache_shape(), POISON_BITS, dtype=np.uint16)


def attention_flops(batch):
    """Algorithmic flop of extend attention: 4*D*Hq per visible (query, key) pair."""
    c = batch.cached_len.astype(np.int64)
    n = batch.new_len.astype(np.int64)
    pairs = int((n * c + n * (n + 1) // 2).sum())
    return 4 * batch.head_dim * batch.num_q_heads * pairs


def attention_bytes(batch, kv_elem_bytes=2):
    """Algorithmic HBM bytes of extend attention: K and V of every visible
    position once per kv head (kv_elem_bytes per element: 2 for a bf16 cache, 1 for
    an 8-bit one), Q in and O out, and the block-table entries."""
    c = batch.cached_len.astype(np.int64)
    n = batch.new_len.astype(np.int64)
    live = n > 0
    kv = int(((c + n) * live).sum()) * 2 * batch.num_kv_heads * batch.head_dim * kv_elem_bytes
    qo = int(n.sum()) * 2 * batch.num_q_heads * batch.head_dim * 2
    bt = int((-(-(c + n) // batch.page_size) * live).sum()) * 4
    return kv + qo + bt


def rope_append_bytes(batch, kv_elem_bytes=2):
    """Algorithmic HBM bytes of rope_append: read q, k, v; write q, K, V (the cache entries
    at kv_elem_bytes per element)."""
    t = batch.total_new
    return t * batch.head_dim * (4 * batch.num_q_heads + 2 * batch.num_kv_heads * (2 + kv_elem_bytes))
