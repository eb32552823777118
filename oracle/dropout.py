"""Dropout masks for the CPU oracle, from the counter-based generator Philox4x32-10.

TEST INFRASTRUCTURE ONLY (same rules as oracle.py: nothing on the product path imports this).

The paper's Transformer workloads train with dropout and the paper shows the primitive as a
module of its Sequential container (Section 4.2, the Sequential listing); it says nothing about how
the random numbers are drawn.  To let a CPU oracle and a GPU kernel agree on every single decision,
both sides draw them from the same counter-based generator (Salmon et al., "Parallel random
numbers: as easy as 1, 2, 3", SC'11: Philox4x32 with 10 rounds), keyed by a 64-bit seed and
addressed by the position of the element, so that no state is shared and any order of evaluation
gives the same mask.  Conventions fixed here (the HIP kernels follow the same ones):

  * key = (seed mod 2^32, seed div 2^32); counter = (c0, c1, c2, c3) as listed per site below;
    one call yields four 32-bit words w0..w3; the element with "column" index n uses word n mod 4
    of the call with c0 = n div 4;
  * an element is KEPT iff its word >= threshold, threshold = min(2^32 - 1, floor(p * 2^32))
    computed in double precision; kept elements are multiplied by 1 / (1 - p);
  * sites: 1 = attention probabilities  (c1 = query i, c0 = key j div 4, c2 = 1, c3 = b*H + h);
           2 = output of the attention projection, before the residual add
           3 = output of the feed-forward activation
           4 = output of the second feed-forward linear, before the residual add
               (sites 2-4: c1 = token row b*T + t, c0 = feature n div 4, c2 = site, c3 = 0);
  * sites 2-4 share one rate (p_hidden), site 1 has its own (p_attn); rate 0 means "no dropout"
    and yields an all-ones mask without drawing anything.
"""
from __future__ import annotations

import numpy as np

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter, key):
    """Philox4x32-10.  counter: four broadcastable uint32 arrays; key: (k0, k1) Python ints.

    Returns four uint32 arrays.  One round:  (hi0, lo0) = M0 * c0,  (hi1, lo1) = M1 * c2 (64-bit
    products split into halves);  c <- (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0);  after each round
    the key is bumped by the Weyl constants (W0, W1) modulo 2^32.
    """
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK32 for c in np.broadcast_arrays(*counter))
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0, k1 = (k0 + _W0) & 0xFFFFFFFF, (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def threshold(p: float) -> int:
    """Words below this value are dropped."""
    if not 0.0 <= p < 1.0:
        raise ValueError("dropout rate must be in [0, 1)")
    return min(2 ** 32 - 1, int(np.floor(np.float64(p) * 4294967296.0)))


def _words(rows, ncols, c2, c3, seed):
    """uint32 [len(rows), ncols]: word (n mod 4) of the call (c0 = n div 4, c1 = row, c2, c3)."""
    n = np.arange(ncols, dtype=np.uint32)
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = philox4x32_10((n[None, :] >> np.uint32(2), np.asarray(rows, np.uint32)[:, None],
                       np.uint32(c2), np.uint32(c3)), key)
    out = np.empty((len(rows), ncols), np.uint32)
    for k in range(4):
        sel = (n & np.uint32(3)) == k
        out[:, sel] = np.broadcast_to(w[k], out.shape)[:, sel]
    return out


def keep_mask_rows(M: int, N: int, site: int, p: float, seed: int) -> np.ndarray:
    """float64 [M, N]: 0 where dropped, 1/(1-p) where kept (sites 2-4)."""
    if p == 0.0:
        return np.ones((M, N))
    keep = _words(np.arange(M), N, site, 0, seed) >= np.uint32(threshold(p))
    return keep / (1.0 - p)


def keep_mask_attention(B: int, H: int, T: int, p: float, seed: int) -> np.ndarray:
    """float64 [B, H, T, T] (query i, key j): 0 where dropped, 1/(1-p) where kept (site 1)."""
    if p == 0.0:
        return np.ones((B, H, T, T))
    out = np.empty((B, H, T, T))
    thr = np.uint32(threshold(p))
    for b in range(B):
        for h in range(H):
            out[b, h] = (_words(np.arange(T), T, 1, b * H + h, seed) >= thr) / (1.0 - p)
    return out


def layer_masks(B, T, D, H, F, p_attn, p_hidden, seed):
    """The four scaled keep masks of one layer call, keyed as layer_forward(masks=...) expects."""
    return {"attn": keep_mask_attention(B, H, T, p_attn, seed),
            "proj": keep_mask_rows(B * T, D, 2, p_hidden, seed).reshape(B, T, D),
            "ffn": keep_mask_rows(B * T, F, 3, p_hidden, seed).reshape(B, T, F),
            "out": keep_mask_rows(B * T, D, 4, p_hidden, seed).reshape(B, T, D)}
