"""TEST INFRASTRUCTURE — reference of the counter-based schedule generator that
the library can run on the device (asynchronous model of the paper, Assumption 3:
who is active, how stale each edge is, which packets are lost, which rows are
sampled).  The schedule of round r is a pure function of (seed, r):

  word(stream, r, e) = Philox4x32-10(counter = (e div 4, stream, r mod 2^32, r div 2^32),
                                     key = (seed mod 2^32, seed div 2^32))[e mod 4]
  active[i]  = word(0, r, i) < floor(p_active[i] * 2^32)
  delay_R[e] = word(1, r, e) mod (d_max + 1)        delay_C[e]: stream 2
  drop_R[e]  = word(3, r, e) < floor(p_drop * 2^32)   drop_C[e]: stream 4
  rows of node i: perm(b), b = 0..B-1, where perm is a keyed bijection of
  [0, samples): a 4-round balanced Feistel network on 2h bits (h = ceil(bits/2),
  bits = bit length of samples-1, at least 1) with cycle walking, its round keys
  the four words of Philox(counter = (i, 5, r lo, r hi)).  Round function on the
  h-bit half R with key K: t = (R * 0x9E3779B1 + K) mod 2^32; t ^= t >> 15;
  t = (t * 0x85EBCA77) mod 2^32; F = t >> (32 - h).

Event-driven form (Algorithm 2 of the paper: exactly one agent i^k per global
iteration k): u = word(6, k, 0); agent i is taken when cdf[i-1] <= u < cdf[i],
cdf[i] = min(floor(2^32 (w_0 + .. + w_i) / sum w), 2^32 - 1) in double precision,
cdf[-1] = 0; u = 2^32 - 1 goes to the last agent if its weight is positive.

Only tests may import this file; it shares no code with the HIP library.
"""
import numpy as np

from .objectives import philox4x32_10

_M32 = np.uint64(0xFFFFFFFF)


def _words(seed, stream, r, count):
    e = np.arange(count, dtype=np.uint64)
    q = e >> np.uint64(2)
    o = philox4x32_10(q, np.full_like(q, stream), np.full_like(q, r & 0xFFFFFFFF), np.full_like(q, (r >> 32) & 0xFFFFFFFF),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    lane = (e & np.uint64(3)).astype(np.int64)
    return np.choose(lane, o).astype(np.uint64)


def _threshold(prob):
    return np.floor(np.asarray(prob, dtype=np.float32).astype(np.float64) * 4294967296.0).astype(np.uint64)


def _feistel(x, keys, h):
    mask = np.uint64((1 << h) - 1)
    L, R = (x >> np.uint64(h)) & mask, x & mask
    for k in keys:
        t = (R * np.uint64(0x9E3779B1) + k) & _M32
        t ^= t >> np.uint64(15)
        t = (t * np.uint64(0x85EBCA77)) & _M32
        F = t >> np.uint64(32 - h)
        L, R = R, L ^ F
    return (L << np.uint64(h)) | R


def sample_rows(seed, r, node, batch, samples):
    q = np.array([node], dtype=np.uint64)
    keys = [k[0] for k in philox4x32_10(q, np.full_like(q, 5), np.full_like(q, r & 0xFFFFFFFF),
                                        np.full_like(q, (r >> 32) & 0xFFFFFFFF), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)]
    bits = max(int(samples - 1).bit_length(), 1)
    h = (bits + 1) // 2
    out = np.empty(batch, dtype=np.int32)
    for b in range(batch):
        x = np.uint64(b)
        while True:
            x = _feistel(x, keys, h)
            if int(x) < samples:
                break
        out[b] = int(x)
    return out


def generate_round(seed, r, n, eR, eC, p_active, d_max, p_drop, batch=0, samples=0):
    thr_a = _threshold(np.broadcast_to(p_active, (n,)))
    thr_d = _threshold(p_drop)
    out = {
        "active": (_words(seed, 0, r, n) < thr_a).astype(np.uint8),
        "delay_R": (_words(seed, 1, r, eR) % np.uint64(d_max + 1)).astype(np.int32),
        "delay_C": (_words(seed, 2, r, eC) % np.uint64(d_max + 1)).astype(np.int32),
        "drop_R": (_words(seed, 3, r, eR) < thr_d).astype(np.uint8),
        "drop_C": (_words(seed, 4, r, eC) < thr_d).astype(np.uint8),
        "batch_idx": None,
    }
    if batch > 0:
        out["batch_idx"] = np.stack([sample_rows(seed, r, i, batch, samples) for i in range(n)])
    return out


def selection_thresholds(weights, n):
    w = np.ones(n, dtype=np.float64) if weights is None else np.asarray(weights, dtype=np.float32).astype(np.float64)
    total = 0.0
    for v in w:          # the same left-to-right sums as a plain loop
        total += float(v)
    cdf, cum = np.empty(n, dtype=np.uint64), 0.0
    for i, v in enumerate(w):
        cum += float(v)
        cdf[i] = min(int(np.floor(cum / total * 4294967296.0)), 0xFFFFFFFF)
    return cdf


def generate_event(seed, k, n, eR, eC, weights, d_max, p_drop, batch=0, samples=0):
    """Schedule of global iteration k: one-hot `active`, the rest as in generate_round."""
    out = generate_round(seed, k, n, eR, eC, 0.0, d_max, p_drop, batch, samples)
    cdf = selection_thresholds(weights, n)
    u = int(_words(seed, 6, k, 1)[0])
    active = np.zeros(n, dtype=np.uint8)
    for i in range(n):
        lo, hi = (int(cdf[i - 1]) if i else 0), int(cdf[i])
        if u >= lo and (u < hi or (i == n - 1 and hi > lo)):
            active[i] = 1
    out["active"] = active
    return out
