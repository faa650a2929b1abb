"""Seeded synthetic workloads for PQTopK scoring (codebook G, sub-item embeddings Psi, sequence embeddings phi).

This module only *draws inputs*: it holds none of the method's arithmetic (no sub-item scores, no item scores,
no top-K).  It is the one module that both the CPU oracle's tests and the HIP path's tests / benchmark import,
so that both sides see identical bytes while sharing no computation.

Shapes follow the paper's notation (Section 2, "Sub-Id based recommendation"; Section 3):
    codes      uint8 [N][m]        row i = sub-ids {g_i1..g_im} of item i          (Eq. 1)
    centroids  fp32  [m][b][d/m]   Psi_k, row j = sub-item embedding psi_{k,j}
    queries    fp32  [B][d]        sequence embeddings phi, one row per user

The paper's own workloads are a Gowalla-shaped catalogue (1,271,638 items, d=512, m=8; Table 1, Section 4) and a
simulation with random model output and random Psi (Section 5, RQ2).  Neither the datasets nor trained RecJPQ
codebooks are available, so every input here is a seeded stand-in of the same shape.

Random numbers come from one counter-based generator, so any element can be drawn independently of the others:

    key(seed, stream) = mix(mix(seed + C0) ^ (stream * C1))
    u64(key, i)       = mix(key + (i + 1) * C0)                   (C0 = 0x9E3779B97F4A7C15, the splitmix64 increment)

with `mix` the splitmix64 output function.  Uniform bytes are the little-endian bytes of consecutive u64 draws;
normals use Box-Muller in float64 on two consecutive draws and are then rounded to fp32.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Tuple

import numpy as np

_MASK = (1 << 64) - 1
_C0 = 0x9E3779B97F4A7C15
_C1 = 0xD1342543DE82EF95

STREAM_CODES = 1
STREAM_CENTROIDS = 2
STREAM_QUERIES = 3
STREAM_ZIPF_PERM = 4
STREAM_DUP_MASK = 5
STREAM_DUP_SRC = 6
STREAM_PLANT = 7
STREAM_CANDIDATES = 8

_CHUNK = 1 << 22  # u64 draws per temporary block


def _mix_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """64-bit key of sub-stream `stream` under `seed`."""
    return _mix_int(_mix_int(seed + _C0) ^ ((stream * _C1) & _MASK))


def u64_at(key: int, start: int, count: int) -> np.ndarray:
    """Draws number start .. start+count-1 of the stream `key`, as uint64."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = idx * np.uint64(_C0) + np.uint64(key)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _unit_open(u: np.ndarray) -> np.ndarray:
    """Map u64 draws to float64 in the open interval (0, 1)."""
    return ((u >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal_f32(key: int, count: int, sigma: float = 1.0) -> np.ndarray:
    """`count` N(0, sigma^2) values as fp32; value i depends only on (key, i)."""
    out = np.empty(count, dtype=np.float32)
    for lo in range(0, count, _CHUNK):
        n = min(_CHUNK, count - lo)
        u = u64_at(key, 2 * lo, 2 * n)
        u1 = _unit_open(u[0::2])
        u2 = _unit_open(u[1::2])
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:lo + n] = (z * sigma).astype(np.float32)
    return out


def centroids(m: int, b: int, d: int, seed: int = 0) -> np.ndarray:
    """Psi as fp32 [m][b][d/m], entries N(0, sigma = d**-0.5) so reconstructed item embeddings have unit norm
    in expectation."""
    if d % m:
        raise ValueError("d must be a multiple of m")
    s = d // m
    return normal_f32(stream_key(seed, STREAM_CENTROIDS), m * b * s, sigma=d ** -0.5).reshape(m, b, s)


def queries(B: int, d: int, seed: int = 0) -> np.ndarray:
    """phi as fp32 [B][d], entries N(0, 1)."""
    return normal_f32(stream_key(seed, STREAM_QUERIES), B * d).reshape(B, d)


def codes_uniform(N: int, m: int, b: int = 256, seed: int = 0) -> np.ndarray:
    """G as uint8 [N][m], each sub-id uniform on [0, b)."""
    if not 1 <= b <= 256:
        raise ValueError("b must be in 1..256")
    key = stream_key(seed, STREAM_CODES)
    total = N * m
    out = np.empty(total, dtype=np.uint8)
    if b == 256:
        words = (total + 7) // 8
        for lo in range(0, words, _CHUNK):
            n = min(_CHUNK, words - lo)
            blk = u64_at(key, lo, n).astype("<u8").view(np.uint8)
            hi = min(total, (lo + n) * 8)
            out[lo * 8:hi] = blk[:hi - lo * 8]
    else:
        for lo in range(0, total, _CHUNK):
            n = min(_CHUNK, total - lo)
            u = u64_at(key, lo, n) >> np.uint64(32)
            out[lo:lo + n] = ((u * np.uint64(b)) >> np.uint64(32)).astype(np.uint8)
    return out.reshape(N, m)


def codes_uniform_u16(N: int, m: int, b: int, seed: int = 0) -> np.ndarray:
    """G as uint16 [N][m] for alphabets of up to 65536 sub-ids per split, each sub-id uniform on [0, b)."""
    if not 1 <= b <= 65536:
        raise ValueError("b must be in 1..65536")
    key = stream_key(seed, STREAM_CODES)
    total = N * m
    out = np.empty(total, dtype=np.uint16)
    for lo in range(0, total, _CHUNK):
        n = min(_CHUNK, total - lo)
        u = u64_at(key, lo, n) >> np.uint64(32)
        out[lo:lo + n] = ((u * np.uint64(b)) >> np.uint64(32)).astype(np.uint16)
    return out.reshape(N, m)


def zipf_cdf(b: int, s: float) -> np.ndarray:
    """Cumulative distribution of P(rank r) proportional to r**-s over ranks 1..b."""
    w = np.arange(1, b + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def zipf_permutations(m: int, b: int, seed: int = 0) -> np.ndarray:
    """Per split, the seeded bijection popularity rank -> sub-id, as uint8 [m][b]."""
    key = stream_key(seed, STREAM_ZIPF_PERM)
    draws = u64_at(key, 0, m * b).reshape(m, b)
    return np.argsort(draws, axis=1, kind="stable").astype(np.uint8 if b <= 256 else np.int64)


def codes_zipf(N: int, m: int, b: int = 256, s: float = 1.1, seed: int = 0) -> np.ndarray:
    """G as uint8 [N][m]; in each split the sub-id popularity follows Zipf(s) (inverse-CDF sampled), and the
    popularity rank is mapped to a sub-id through a seeded per-split permutation."""
    key = stream_key(seed, STREAM_CODES)
    cdf = zipf_cdf(b, s)
    perm = zipf_permutations(m, b, seed)
    total = N * m
    out = np.empty(total, dtype=np.uint8)
    split_of = np.arange(m, dtype=np.int64)
    for lo in range(0, total, _CHUNK):
        n = min(_CHUNK, total - lo)
        u = _unit_open(u64_at(key, lo, n))
        rank = np.minimum(np.searchsorted(cdf, u, side="left"), b - 1)
        k = split_of[(np.arange(lo, lo + n, dtype=np.int64)) % m]
        out[lo:lo + n] = perm[k, rank]
    return out.reshape(N, m)


def duplicate_rows(codes: np.ndarray, fraction: float = 0.05, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Force exact score ties: a seeded `fraction` of the ids i >= 1 get G[i] = G[j] for a seeded j < i.

    Returns (codes, src) where src[i] is the id whose original row item i now carries (src[i] == i if untouched).
    Copies are resolved through chains, so the result equals applying the copies in increasing order of i."""
    N = codes.shape[0]
    ids = np.arange(N, dtype=np.int64)
    mask_draw = _unit_open(u64_at(stream_key(seed, STREAM_DUP_MASK), 0, N))
    src_draw = u64_at(stream_key(seed, STREAM_DUP_SRC), 0, N)
    is_dup = (mask_draw < fraction) & (ids > 0)
    j = (src_draw % np.maximum(ids, 1).astype(np.uint64)).astype(np.int64)
    src = np.where(is_dup, j, ids)
    while True:  # pointer jumping; every hop strictly lowers the id, so this ends
        nxt = src[src]
        if np.array_equal(nxt, src):
            break
        src = nxt
    return np.ascontiguousarray(codes[src]), src


def plant_ids(N: int, count: int, seed: int = 0) -> np.ndarray:
    """`count` distinct seeded item ids in [0, N), ascending."""
    if count > N:
        raise ValueError("count > N")
    key = stream_key(seed, STREAM_PLANT)
    got: list = []
    seen = set()
    start = 0
    while len(got) < count:
        for v in (u64_at(key, start, 2 * count) % np.uint64(N)).tolist():
            if v not in seen:
                seen.add(v)
                got.append(v)
                if len(got) == count:
                    break
        start += 2 * count
    return np.sort(np.asarray(got, dtype=np.int64))


def candidate_list(N: int, count: int, seed: int = 0, ascending: bool = False) -> np.ndarray:
    """Candidate list V for Algorithm 1: `count` distinct seeded item ids in [0, N) as int32, in a seeded random
    order (or ascending).  Drawn as the first `count` entries of a seeded permutation of the catalogue."""
    if count > N:
        raise ValueError("count > N")
    key = stream_key(seed, STREAM_CANDIDATES)
    order = np.argsort(u64_at(key, 0, N), kind="stable")[:count].astype(np.int32)
    return np.sort(order) if ascending else order


def codes_uniform_device(N: int, m: int, b: int = 256, seed: int = 0):
    """Uniform sub-ids drawn on the GPU (torch's seeded device generator) as a uint8 [N][m] device tensor: for
    catalogues too large to draw on the host in reasonable time (the catalogue-size sweep).  Not the same stream
    as codes_uniform(); whoever checks results copies the tensor back."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randint(0, b, (N, m), dtype=torch.uint8, device="cuda", generator=g)


def codes_uniform_u16_device(N: int, m: int, b: int, seed: int = 0):
    """codes_uniform_device() for alphabets of up to 65536 sub-ids: a uint16 [N][m] device tensor."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = torch.empty((N, m), dtype=torch.uint16, device="cuda")
    step = max(1, (1 << 26) // m)                              # drawn in slices: the int32 staging stays small
    for lo in range(0, N, step):
        n = min(step, N - lo)
        out[lo:lo + n] = torch.randint(0, b, (n, m), dtype=torch.int32, device="cuda", generator=g).to(torch.uint16)
    return out


def plant_rows(codes: np.ndarray, ids: np.ndarray, row: np.ndarray) -> np.ndarray:
    """Overwrite the code rows of `ids` with `row` (in place); the caller decides which row to plant."""
    codes[np.asarray(ids, dtype=np.int64)] = np.asarray(row, dtype=np.uint8)[None, :]
    return codes


@dataclasses.dataclass(frozen=True)
class Config:
    """One named workload: catalogue size N, embedding dim d, m splits, b sub-ids per split, batch sizes, K."""
    name: str
    N: int
    d: int
    m: int
    b: int
    batches: Tuple[int, ...]
    K: int
    codes: str  # "uniform" | "zipf" | "uniform+dup"
    seed: int = 0


CONFIGS: Dict[str, Config] = {
    c.name: c for c in (
        Config("tiny", 10_000, 64, 4, 256, (1,), 10, "uniform"),
        Config("large", 1_280_000, 512, 8, 256, (1, 64), 10, "uniform"),       # Gowalla-shaped (Table 1)
        Config("serving", 1_280_000, 512, 8, 256, (1024,), 100, "zipf"),
        Config("finer", 5_000_000, 512, 16, 256, (16,), 10, "uniform+dup"),
        Config("huge", 50_000_000, 512, 8, 256, (1, 32), 10, "uniform"),       # RQ2-style simulated catalogue
    )
}


def make(cfg: Config, B: int | None = None, N: int | None = None):
    """Draw (codes, centroids, queries) for a config; B / N override the config's batch / catalogue size."""
    B = cfg.batches[0] if B is None else B
    N = cfg.N if N is None else N
    if cfg.codes == "zipf":
        G = codes_zipf(N, cfg.m, cfg.b, 1.1, cfg.seed)
    else:
        G = codes_uniform(N, cfg.m, cfg.b, cfg.seed)
        if cfg.codes == "uniform+dup":
            G, _ = duplicate_rows(G, 0.05, cfg.seed)
    return G, centroids(cfg.m, cfg.b, cfg.d, cfg.seed), queries(B, cfg.d, cfg.seed)
