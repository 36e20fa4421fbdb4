"""Seeded synthetic inputs for the KNN-softmax path (class weights, features, labels, neighbour lists).

This module only produces *inputs*: it holds none of the method's arithmetic (no logits, no softmax, no
similarity ranking).  Both the CPU oracle's tests and the HIP path's tests/bench draw their inputs from
here so that the two sides see the same bits.

Generator: a counter-based stream.  Element `e` of tensor `tid` under `seed` is derived from
splitmix64 hashes of a 64-bit counter keyed by (seed, tid, e); normals come from Box-Muller in fp64.
Any sub-range of a tensor can therefore be generated independently (used to build big matrices in
row chunks on several threads) and always yields the same values.

The paper's data (private SKU-1M/10M/100M product images) is not available; these inputs stand in for
it with the shapes the paper gives (feature dimension 512, one GPU's share of 100 M classes over 256
GPUs, active set about 10 % of the shard).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

# tensor ids (any distinct small integers)
TID_W, TID_X, TID_LABELS, TID_PERM, TID_CENTRES, TID_NOISE, TID_GRAPH, TID_DW, TID_MISC = range(1, 10)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output step applied element-wise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x.astype(_U64, copy=True)
        z += _GOLD
        z ^= z >> _U64(30)
        z *= _M1
        z ^= z >> _U64(27)
        z *= _M2
        z ^= z >> _U64(31)
    return z


def _base(seed: int, tid: int) -> np.uint64:
    k = splitmix64(np.array([(int(seed) & 0xFFFFFFFF) * 0x100000001B3 + int(tid) * 0x9E3779B1], dtype=_U64))
    return splitmix64(k)[0]


def raw_u64(seed: int, tid: int, start: int, count: int, lane: int = 0) -> np.ndarray:
    """uint64 hash for elements [start, start+count) of tensor `tid`; `lane` selects independent streams."""
    with np.errstate(over="ignore"):
        ctr = (np.arange(start, start + count, dtype=_U64) * _U64(4) + _U64(lane)) ^ _base(seed, tid)
    return splitmix64(ctr)


def uniform01(seed: int, tid: int, start: int, count: int, lane: int = 0) -> np.ndarray:
    """fp64 uniforms in (0, 1): (top 53 bits + 0.5) / 2^53."""
    h = raw_u64(seed, tid, start, count, lane)
    return ((h >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, tid: int, start: int, count: int) -> np.ndarray:
    """fp64 N(0,1) by Box-Muller from two uniforms per element."""
    u1 = uniform01(seed, tid, start, count, 0)
    u2 = uniform01(seed, tid, start, count, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


# ---------------------------------------------------------------------------------------------
# bf16 helpers (data preparation only: round-to-nearest-even of fp32 to the bf16 grid)
# ---------------------------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns (round to nearest even; inputs must be finite)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 array rounded onto the bf16 grid, returned as fp32."""
    return bf16_to_f32(bf16_bits(x))


# ---------------------------------------------------------------------------------------------
# matrices
# ---------------------------------------------------------------------------------------------
def _n_threads() -> int:
    return max(1, min(16, (os.cpu_count() or 1)))


def _chunked_rows(fn, n_rows: int, D: int, out: np.ndarray, rows_per_chunk: int = 8192) -> None:
    chunks = [(r0, min(n_rows, r0 + rows_per_chunk)) for r0 in range(0, n_rows, rows_per_chunk)]
    if len(chunks) <= 1:
        for r0, r1 in chunks:
            out[r0:r1] = fn(r0, r1)
        return

    def work(c):
        out[c[0]:c[1]] = fn(c[0], c[1])

    with ThreadPoolExecutor(max_workers=_n_threads()) as ex:
        list(ex.map(work, chunks))


def unit_rows(seed: int, tid: int, n_rows: int, D: int, bf16: bool = False) -> np.ndarray:
    """[n_rows, D] fp32: rows i.i.d. N(0,1), L2-normalised in fp64, rounded to fp32 (then to the bf16 grid
    when `bf16`).  After bf16 rounding the rows are unit only to about 2^-9."""
    out = np.empty((n_rows, D), dtype=np.float32)

    def fn(r0, r1):
        g = normal(seed, tid, r0 * D, (r1 - r0) * D).reshape(r1 - r0, D)
        g /= np.sqrt((g * g).sum(axis=1, keepdims=True))
        f = g.astype(np.float32)
        return bf16_round(f) if bf16 else f

    _chunked_rows(fn, n_rows, D, out)
    return out


def clustered_rows(seed: int, n_rows: int, D: int, n_centres: int = 4096, noise: float = 0.3,
                   bf16: bool = False) -> np.ndarray:
    """Rows = centre[c mod n_centres] + noise * N(0,1)/sqrt(D)-scaled perturbation, L2-normalised.
    Gives heavily overlapping neighbour lists, like trained class weights of similar products."""
    centres = unit_rows(seed, TID_CENTRES, min(n_centres, n_rows), D).astype(np.float64)
    nc = centres.shape[0]
    out = np.empty((n_rows, D), dtype=np.float32)

    def fn(r0, r1):
        g = normal(seed, TID_NOISE, r0 * D, (r1 - r0) * D).reshape(r1 - r0, D)
        g /= np.sqrt((g * g).sum(axis=1, keepdims=True))
        v = centres[np.arange(r0, r1) % nc] + noise * g
        v /= np.sqrt((v * v).sum(axis=1, keepdims=True))
        f = v.astype(np.float32)
        return bf16_round(f) if bf16 else f

    _chunked_rows(fn, n_rows, D, out)
    return out


def features_near_labels(seed: int, W: np.ndarray, labels: np.ndarray, sigma: float = 0.5,
                         bf16: bool = False) -> np.ndarray:
    """Features that look like a partly trained model's: x_i = normalise(w_{y_i} + sigma * unit noise).
    Makes the softmax peaky (target logit near the scale s), the hard regime for the fused softmax."""
    B, D = labels.shape[0], W.shape[1]
    g = normal(seed, TID_X, 0, B * D).reshape(B, D)
    g /= np.sqrt((g * g).sum(axis=1, keepdims=True))
    v = W[labels].astype(np.float64) + sigma * g
    v /= np.sqrt((v * v).sum(axis=1, keepdims=True))
    f = v.astype(np.float32)
    return bf16_round(f) if bf16 else f


# ---------------------------------------------------------------------------------------------
# labels
# ---------------------------------------------------------------------------------------------
def labels_uniform(seed: int, B: int, C: int) -> np.ndarray:
    u = uniform01(seed, TID_LABELS, 0, B)
    return np.minimum((u * C).astype(np.int64), C - 1).astype(np.int32)


def class_permutation(seed: int, C: int) -> np.ndarray:
    """Seeded permutation of [0, C): argsort of per-class hashes (ties broken by index, stable)."""
    return np.argsort(raw_u64(seed, TID_PERM, 0, C), kind="stable").astype(np.int32)


def labels_zipf(seed: int, B: int, C: int, alpha: float = 1.1) -> np.ndarray:
    """Labels with p(rank r) proportional to r^-alpha, r = 1..C, rank -> class through a seeded
    permutation; sampling by inverse CDF on an fp64 cumulative table."""
    p = np.arange(1, C + 1, dtype=np.float64) ** (-alpha)
    cdf = np.cumsum(p)
    cdf /= cdf[-1]
    u = uniform01(seed, TID_LABELS, 0, B)
    rank = np.minimum(np.searchsorted(cdf, u, side="left"), C - 1)
    return class_permutation(seed, C)[rank].astype(np.int32)


# ---------------------------------------------------------------------------------------------
# neighbour lists that are inputs (not computed from W): used where a brute-force graph of the
# full class matrix is out of the CPU oracle's reach, and to exercise selection structure
# ---------------------------------------------------------------------------------------------
def graph_synthetic(seed: int, C: int, K: int, locality: int = 64, empty_frac: float = 0.0) -> np.ndarray:
    """int32 [C, K]: for class c, K distinct ids != c.  Half of each list is drawn from a window of
    `locality`*K ids around c (so lists of nearby classes overlap, as in a real KNN graph of clustered
    weights), the rest uniformly over all classes.  `empty_frac` > 0 replaces that share of trailing
    slots by -1 (empty), as a compressed list would have.  Requires K <= C - 1."""
    assert 1 <= K <= C - 1
    G = np.empty((C, K), dtype=np.int32)
    rows_per = max(1, (1 << 22) // max(K, 1))
    win = max(2 * K + 2, locality * K)
    for r0 in range(0, C, rows_per):
        r1 = min(C, r0 + rows_per)
        n = r1 - r0
        c = np.arange(r0, r1, dtype=np.int64)[:, None]
        h = raw_u64(seed, TID_GRAPH, r0 * K, n * K).reshape(n, K)
        col = np.arange(K)[None, :]
        near = (c + 1 + (h % _U64(win)).astype(np.int64) - win // 2) % C
        far = (h >> _U64(20)).astype(np.int64) % C
        cand = np.where(col % 2 == 0, near, far)
        # repair collisions (self or duplicate within the row) deterministically by linear probing
        srt = np.sort(cand, axis=1)
        bad = (srt[:, 1:] == srt[:, :-1]).any(axis=1) | (cand == c).any(axis=1)
        for i in np.nonzero(bad)[0]:
            row = cand[i]
            seen = {int(c[i, 0])}
            for k in range(K):
                v = int(row[k])
                while v in seen:
                    v = (v + 1) % C
                seen.add(v)
                row[k] = v
        G[r0:r1] = cand.astype(np.int32)
    if empty_frac > 0.0:
        u = uniform01(seed, TID_GRAPH, 0, C, 2)
        n_empty = np.minimum((u * empty_frac * 2 * K).astype(np.int64), K - 1)
        mask = np.arange(K)[None, :] >= (K - n_empty)[:, None]
        G[mask] = -1
    return G


def graph_synthetic_rows(seed: int, C: int, K: int, rows: np.ndarray, locality: int = 64) -> np.ndarray:
    """The rows `rows` of graph_synthetic(seed, C, K, locality) without building the whole array."""
    rows = np.asarray(rows, dtype=np.int64)
    win = max(2 * K + 2, locality * K)
    out = np.empty((rows.shape[0], K), dtype=np.int32)
    for i, c in enumerate(rows):
        h = raw_u64(seed, TID_GRAPH, int(c) * K, K)
        near = (int(c) + 1 + (h % _U64(win)).astype(np.int64) - win // 2) % C
        far = (h >> _U64(20)).astype(np.int64) % C
        cand = np.where(np.arange(K) % 2 == 0, near, far)
        seen = {int(c)}
        for k in range(K):
            v = int(cand[k])
            while v in seen:
                v = (v + 1) % C
            seen.add(v)
            cand[k] = v
        out[i] = cand
    return out


def graph_all_others(C: int) -> np.ndarray:
    """int32 [C, C-1]: row c lists every other class in ascending order (the K = C-1 case in which the
    active set is the whole class set)."""
    G = np.empty((C, C - 1), dtype=np.int32)
    ar = np.arange(C, dtype=np.int32)
    for c in range(C):
        G[c, :c] = ar[:c]
        G[c, c:] = ar[c + 1:]
    return G


def grad_rows(seed: int, n: int, D: int) -> np.ndarray:
    """fp32 [n, D] N(0, 1e-2) stand-in for weight-gradient rows (input of the weight update)."""
    out = np.empty((n, D), dtype=np.float32)
    _chunked_rows(lambda r0, r1: (0.1 * normal(seed, TID_DW, r0 * D, (r1 - r0) * D)).reshape(r1 - r0, D).astype(np.float32),
                  n, D, out)
    return out


# ---------------------------------------------------------------------------------------------
# the named workloads (shapes of the five configurations this build is measured on)
# ---------------------------------------------------------------------------------------------
CONFIGS = {
    # name: C, D, B, K, M, bf16 inputs, label law
    "tiny": dict(C=10_000, D=128, B=64, K=8, M=1_024, bf16=False, labels="uniform", scale=30.0, seed=0),
    "small": dict(C=100_000, D=256, B=256, K=16, M=4_096, bf16=True, labels="uniform", scale=30.0, seed=0),
    "shard390k": dict(C=390_625, D=512, B=1_024, K=32, M=32_768, bf16=True, labels="zipf", scale=30.0, seed=0),
    "shard390k_uniform": dict(C=390_625, D=512, B=1_024, K=32, M=32_768, bf16=True, labels="uniform",
                              scale=30.0, seed=0),
    # the headline shape with clustered class weights (centre[c mod 4096] + 0.3 noise): neighbour lists overlap
    # heavily, as those of trained weights of similar products do
    "shard390k_clustered": dict(C=390_625, D=512, B=1_024, K=32, M=32_768, bf16=True, labels="zipf", scale=30.0,
                                seed=0, weights="clustered"),
    "dense1m": dict(C=1_000_000, D=512, B=2_048, K=64, M=131_072, bf16=True, labels="uniform", scale=30.0,
                    seed=0),
}


def make_labels(cfg: dict, seed: int | None = None) -> np.ndarray:
    seed = cfg["seed"] if seed is None else seed
    if cfg["labels"] == "zipf":
        return labels_zipf(seed, cfg["B"], cfg["C"], 1.1)
    return labels_uniform(seed, cfg["B"], cfg["C"])


def make_WX(cfg: dict, seed: int | None = None):
    """(W [C,D] fp32, X [B,D] fp32), on the bf16 grid when cfg['bf16']."""
    seed = cfg["seed"] if seed is None else seed
    if cfg.get("weights") == "clustered":
        W = clustered_rows(seed, cfg["C"], cfg["D"], bf16=cfg["bf16"])
    else:
        W = unit_rows(seed, TID_W, cfg["C"], cfg["D"], bf16=cfg["bf16"])
    X = unit_rows(seed, TID_X, cfg["B"], cfg["D"], bf16=cfg["bf16"])
    return W, X


# ---------------------------------------------------------------------------------------------
# inputs of the layer-wise top-k sparsification (Section 3.3): a set of gradient tensors with the
# sizes of a ResNet-50's parameters (the feature-extraction net of the paper's experiments)
# ---------------------------------------------------------------------------------------------
TID_GRAD_SET = 20


def resnet50_tensor_sizes(num_classes: int = 1000) -> list[int]:
    """Element counts of the parameter tensors of a ResNet-50 (convolutions, batch-norm scale and shift,
    classifier), in network order: 161 tensors, 25,557,032 elements for 1,000 classes."""
    sizes = [64 * 3 * 7 * 7, 64, 64]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            sizes += [planes * inplanes, planes, planes]          # 1x1 reduce + bn
            sizes += [planes * planes * 9, planes, planes]         # 3x3 + bn
            sizes += [4 * planes * planes, 4 * planes, 4 * planes]  # 1x1 expand + bn
            if b == 0:
                sizes += [4 * planes * inplanes, 4 * planes, 4 * planes]  # projection shortcut + bn
            inplanes = 4 * planes
    sizes += [num_classes * 2048, num_classes]
    return sizes


def grad_tensor_set(seed: int, sizes, zero_every: int = 5) -> tuple[np.ndarray, np.ndarray]:
    """(flat fp32 array holding the tensors back to back, int64 offsets [T + 1]).  Tensor t is N(0, s_t^2) with
    s_t = 1e-3 * 2^(t mod 7 - 3); every `zero_every`-th tensor has its second eighth set to exactly zero and
    its third eighth rounded to multiples of s_t / 4 (dead units and repeated values: ties)."""
    offs = np.zeros(len(sizes) + 1, dtype=np.int64)
    offs[1:] = np.cumsum(np.asarray(sizes, dtype=np.int64))
    total = int(offs[-1])
    g = np.empty(total, dtype=np.float32)
    step = 1 << 22
    for s0 in range(0, total, step):
        s1 = min(total, s0 + step)
        g[s0:s1] = normal(seed, TID_GRAD_SET, s0, s1 - s0).astype(np.float32)
    for t, n in enumerate(sizes):
        a, sc = int(offs[t]), np.float32(1e-3 * 2.0 ** (t % 7 - 3))
        g[a:a + n] *= sc
        if zero_every and t % zero_every == 0 and n >= 8:
            e = n // 8
            g[a + e:a + 2 * e] = 0.0
            q = sc / np.float32(4)
            g[a + 2 * e:a + 3 * e] = np.round(g[a + 2 * e:a + 3 * e] / q) * q
    return g, offs


def topk_counts(sizes, density: float = 1e-3) -> np.ndarray:
    """k per tensor at the given density (99.9 % sparsity by default), at least 1."""
    return np.maximum(1, np.floor(np.asarray(sizes, dtype=np.float64) * density)).astype(np.int32)
