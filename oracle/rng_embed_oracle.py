"""CPU oracle for the two pieces either side of the layer-shard path: the model-parallel random number streams that
drive dropout, and the vocabulary-parallel input embedding.

TEST INFRASTRUCTURE ONLY.  Like oracle/layer_oracle.py this file is the checker, not the product: only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import it.  It shares no code with the
HIP path and imports nothing from it.

What it defines.

* Random streams (Appendix B.2 of the paper, "Model Parallel Random Number Generation"): dropout outside the
  model-parallel regions (embedding output, the two block outputs before their residual adds) must use the SAME
  pattern on every worker, so those sites draw from a stream seeded identically everywhere; dropout inside a
  model-parallel region (the attention probabilities of a worker's local heads) must differ between workers, so it
  draws from a second stream whose seed is unique per worker.  The paper fixes neither the generator nor the seed
  derivation.  Reading taken: both streams are the counter-based Philox4x32-10 generator (Salmon, Moraes, Dror, Shaw:
  "Parallel random numbers: as easy as 1, 2, 3", SC'11) keyed with a 64-bit seed; the replicated stream's seed is the
  base seed, worker r's model-parallel seed is base + 1 + r (mod 2^64).  Element e of a dropout site (row-major
  index in the tensor the WORKER holds) takes word ``e mod 4`` of the block with counter
  ``(lo32(e div 4), hi32(e div 4), lo32(offset), hi32(offset))``, where the 64-bit ``offset`` names the site
  (layer, call, training step) and is chosen by the caller; the element is KEPT iff that 32-bit word is >=
  ``floor(p * 2^32)`` with p the drop probability as a float32 value.  The decision is integer work: bit-exact.

* Vocabulary-parallel input embedding (Section 3): the embedding table shares its weights with the output embedding
  ``E [H, v]`` and is split along the vocabulary like it; worker r produces ``E_r[:, id - v0]`` for the ids inside
  its range and zeros elsewhere, the reduction ``g`` sums the partials, then the (replicated) position embedding is
  added and the replicated-stream dropout applied.  The backward pass scatters the gradient rows back into the
  columns of ``dE_r`` (adding up repeated ids), on top of the output embedding's gradient (tied weights).

Pins (tests/test_rng_embed_pins.py, CPU): the published Philox4x32-10 known-answer vectors, a scalar re-derivation of
one block by pure-Python integer arithmetic, keep-rate statistics, stream identity / distinctness rules, one-hot
matmul and library (torch embedding + autograd) equivalents of the lookup and its gradient, and the sharding
invariant (sum over shards == unsharded lookup, exactly).
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64
U32 = np.uint32
U64 = np.uint64

_M0 = U64(0xD2511F53)
_M1 = U64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = U64(0xFFFFFFFF)

STREAM_REPLICATED = 0      # same pattern on every model-parallel worker
STREAM_MODEL_PARALLEL = 1  # pattern unique to worker r


def philox4x32_10(counter: np.ndarray, key: Sequence[int]) -> np.ndarray:
    """Philox4x32 with 10 rounds.  counter: [..., 4] uint32; key: two 32-bit integers.  Returns [..., 4] uint32.

    One round maps (c0, c1, c2, c3) to (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0)); the key is
    advanced by the Weyl constants (W0, W1) before every round but the first."""
    c = np.asarray(counter, dtype=U32)
    c0, c1, c2, c3 = (c[..., i].astype(U64) for i in range(4))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> U64(32), p0 & _MASK32
        hi1, lo1 = p1 >> U64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ U64(k0), lo1, hi0 ^ c3 ^ U64(k1), lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(U32)


def stream_seed(base_seed: int, stream: int, r: int) -> int:
    """64-bit seed of a dropout stream on worker r (Appendix B.2): identical on all workers for the replicated stream,
    unique per worker for the model-parallel stream."""
    base_seed &= 0xFFFFFFFFFFFFFFFF
    if stream == STREAM_REPLICATED:
        return base_seed
    if stream == STREAM_MODEL_PARALLEL:
        if r < 0:
            raise ValueError("worker index must be non-negative")
        return (base_seed + 1 + r) & 0xFFFFFFFFFFFFFFFF
    raise ValueError("unknown stream")


def drop_threshold(p_drop: float) -> int:
    """floor(p * 2^32) for the float32 value of p (0 <= p < 1): an element is kept iff its random word >= this."""
    p32 = float(np.float32(p_drop))
    if not (0.0 <= p32 < 1.0):
        raise ValueError("drop probability must be in [0, 1)")
    return int(np.floor(p32 * 4294967296.0))


def random_words(seed: int, offset: int, n: int, first: int = 0) -> np.ndarray:
    """The 32-bit words of elements first .. first+n-1 of the site named ``offset`` in the stream seeded ``seed``."""
    e = np.arange(first, first + n, dtype=U64)
    blk = e >> U64(2)
    ctr = np.empty((n, 4), U32)
    ctr[:, 0] = (blk & _MASK32).astype(U32)
    ctr[:, 1] = (blk >> U64(32)).astype(U32)
    ctr[:, 2] = offset & 0xFFFFFFFF
    ctr[:, 3] = (offset >> 32) & 0xFFFFFFFF
    out = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    return out[np.arange(n), (e & U64(3)).astype(np.int64)]


def keep_mask(seed: int, offset: int, shape: Tuple[int, ...], p_drop: float) -> np.ndarray:
    """Boolean keep mask of a dropout site: elements in row-major order of ``shape``."""
    n = int(np.prod(shape))
    return (random_words(seed, offset, n) >= U32(drop_threshold(p_drop))).reshape(shape)


def layer_dropout_masks(b: int, s: int, H: int, h: int, p: int, base_seed: int, offsets: Dict[str, int],
                        p_attn: float, p_hidden: float) -> Dict[str, object]:
    """The keep masks of one layer in UNSHARDED coordinates, assembled by the method's rule.

    keep1 / keep2 ([T, H], the dropouts before the two residual adds) come from the replicated stream; the attention
    mask of global head k comes from the model-parallel stream of the worker r = k div (h/p) that owns it, at that
    worker's local index ((batch * h_l + local head) * s + i) * s + j.  offsets: {"attn", "hidden1", "hidden2"}.
    Returns the ``drop`` entry the layer oracle accepts."""
    hl = h // p
    T = b * s
    rep = stream_seed(base_seed, STREAM_REPLICATED, 0)
    keep_attn = np.empty((b, h, s, s), bool)
    for r in range(p):
        local = keep_mask(stream_seed(base_seed, STREAM_MODEL_PARALLEL, r), offsets["attn"], (b, hl, s, s), p_attn)
        keep_attn[:, r * hl:(r + 1) * hl] = local
    return {"keep_attn": keep_attn,
            "keep1": keep_mask(rep, offsets["hidden1"], (T, H), p_hidden),
            "keep2": keep_mask(rep, offsets["hidden2"], (T, H), p_hidden),
            "p_attn": float(np.float32(p_attn)), "p_hidden": float(np.float32(p_hidden))}


# --------------------------------------------------------------------------- input embedding
def embedding_fwd(E, ids, pos=None, keep=None, p_drop: float = 0.0):
    """X0[t, :] = dropout(E[:, ids[t]] + pos[t mod s, :]).  E: [H, V] (the output embedding's matrix, tied);
    ids: [b, s] int; pos: [s, H] or None; keep: [T, H] bool or None.  Returns X0 [T, H]."""
    E = np.asarray(E, F64)
    ids = np.asarray(ids)
    b, s = ids.shape
    x = E[:, ids.reshape(-1)].T.copy()
    if pos is not None:
        x = x + np.tile(np.asarray(pos, F64), (b, 1))
    if keep is not None:
        x = np.where(np.asarray(keep, bool), x, 0.0) / (1.0 - p_drop)
    return x


def embedding_bwd(dX0, ids, V: int, s: int, keep=None, p_drop: float = 0.0):
    """Gradients of embedding_fwd: dE [H, V] with dE[:, v] = sum over tokens with id v of the (dropout-masked) rows
    of dX0, and dpos [s, H] = sum over the batch.  Plain loops: this is the definition."""
    d = np.asarray(dX0, F64)
    if keep is not None:
        d = np.where(np.asarray(keep, bool), d, 0.0) / (1.0 - p_drop)
    T, H = d.shape
    flat = np.asarray(ids).reshape(-1)
    dE = np.zeros((H, V), F64)
    dpos = np.zeros((s, H), F64)
    for t in range(T):
        dE[:, flat[t]] += d[t]
        dpos[t % s] += d[t]
    return dE, dpos


def embedding_sharded(E, ids, p: int):
    """The vocabulary-parallel lookup written out: per-shard partials [p][T, H] (zeros for ids outside the shard's
    range) whose sum -- the reduction g -- is the unsharded lookup."""
    E = np.asarray(E, F64)
    H, V = E.shape
    flat = np.asarray(ids).reshape(-1)
    Vl = V // p
    parts = []
    for r in range(p):
        v0, v1 = r * Vl, (r + 1) * Vl
        inside = (flat >= v0) & (flat < v1)
        part = np.zeros((flat.size, H), F64)
        part[inside] = E[:, v0:v1][:, flat[inside] - v0].T
        parts.append(part)
    return parts
