"""Seeded synthetic inputs for the hot-embedding path (inputs only, no method arithmetic).

Everything here is *data generation*: sparse-index streams with Zipf-skewed
popularity, bag lengths, upstream gradients and procedural table weights.  Both
the CPU oracle's tests and the HIP path's tests/bench feed on the same tensors
produced here; nothing in this module computes a histogram, a remap, a pooled
sum or an update.

All draws come from one counter-based generator (a 64-bit mixing function of
``(seed, stream, counter)``), so a value depends only on its position in the
stream, never on chunking, thread count or device.  The integer parts are
bit-identical on CPU and GPU tensors; the Zipf inversion uses fp64 ``pow`` and
may differ in the last ulp between devices, so a test always generates once and
hands the *same* tensor to both implementations.

The workloads stand in for the paper's datasets (Table 2: Taobao, Criteo Kaggle,
Criteo Terabyte, Avazu), which are not available: same table counts, row
dimensions, one-hot vs. multi-hot structure and popularity skew (Sec. 1: a few
per cent of the rows receive most of the accesses), but no record of any of them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence

import torch

SEED = 20210300686  # paper id, used as the master seed everywhere

_M64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int (mod 2^64) -> the same bit pattern as a signed 64-bit value."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLD = _s64(0x9E3779B97F4A7C15)
_MULA = _s64(0xBF58476D1CE4E5B9)
_MULB = _s64(0x94D049BB133111EB)
_MULC = _s64(0xD1B54A32D192ED03)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """The splitmix64 output function on int64 bit patterns (wrap-around multiply)."""
    x = x ^ _lsr(x, 30)
    x = x * _MULA
    x = x ^ _lsr(x, 27)
    x = x * _MULB
    x = x ^ _lsr(x, 31)
    return x


def mix64_int(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x


def stream_key(seed: int, *ids: int) -> int:
    """Fold a seed and a tuple of small ids into one 64-bit stream key."""
    k = mix64_int(seed)
    for i in ids:
        k = mix64_int(k ^ ((0x9E3779B97F4A7C15 * (i + 1)) & _M64))
    return k


def hash_counter(key: int, counter: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits for every counter value under a stream key."""
    return mix64(counter * _MULC + _s64(key))


def uniform01(key: int, counter: torch.Tensor) -> torch.Tensor:
    """fp64 uniforms in [0, 1) (53 random bits each)."""
    h = hash_counter(key, counter)
    return _lsr(h, 11).to(torch.float64) * (1.0 / (1 << 53))


# --------------------------------------------------------------------------------------
# Zipf ranks: exact bounded Zipf by rejection-inversion (Hoermann & Derflinger, 1996)
# --------------------------------------------------------------------------------------
class _ZipfRI:
    def __init__(self, n: int, s: float):
        assert n >= 1 and s > 0
        self.n, self.s = n, s
        self.log_form = abs(1.0 - s) < 1e-12
        self.h_x1 = self._H_f(1.5) - 1.0
        self.h_n = self._H_f(n + 0.5)
        self.thr = 2.0 - self._Hinv_f(self._H_f(2.5) - 2.0 ** (-s))

    def _H_f(self, x: float) -> float:
        return math.log(x) if self.log_form else (x ** (1.0 - self.s) - 1.0) / (1.0 - self.s)

    def _Hinv_f(self, y: float) -> float:
        return math.exp(y) if self.log_form else (1.0 + (1.0 - self.s) * y) ** (1.0 / (1.0 - self.s))

    def H(self, x: torch.Tensor) -> torch.Tensor:
        if self.log_form:
            return torch.log(x)
        return (torch.pow(x, 1.0 - self.s) - 1.0) / (1.0 - self.s)

    def Hinv(self, y: torch.Tensor) -> torch.Tensor:
        if self.log_form:
            return torch.exp(y)
        return torch.pow(1.0 + (1.0 - self.s) * y, 1.0 / (1.0 - self.s))

    def draw(self, u01: torch.Tensor):
        """One attempt per element: returns (rank in [1,n], accepted mask)."""
        u = self.h_n + u01 * (self.h_x1 - self.h_n)
        x = self.Hinv(u)
        k = torch.clamp(torch.floor(x + 0.5), 1.0, float(self.n))
        acc = (k - x <= self.thr) | (u >= self.H(k + 0.5) - torch.pow(k, -self.s))
        return k.to(torch.int64), acc


def _zipf_at(z: _ZipfRI, key: int, pos: torch.Tensor) -> torch.Tensor:
    """Ranks for the given stream positions; attempt ``a`` of position ``p`` uses
    counter ``p*64 + a``, so attempts of different elements never collide."""
    n = pos.numel()
    out = torch.empty(n, dtype=torch.int64, device=pos.device)
    todo = torch.arange(n, dtype=torch.int64, device=pos.device)
    attempt = 0
    while todo.numel() > 0:
        k, acc = z.draw(uniform01(key, pos[todo] * 64 + attempt))
        out[todo[acc]] = k[acc]
        todo = todo[~acc]
        attempt += 1
        if attempt >= 64:  # probability of reaching this is astronomically small
            out[todo] = 1
            break
    return out


def zipf_ranks(n: int, n_rows: int, s: float, key: int, start: int = 0,
               device: str | torch.device = "cpu") -> torch.Tensor:
    """``n`` ranks in [1, n_rows] with P(k) proportional to k^-s; element i depends on
    its stream position ``start + i`` only."""
    pos = torch.arange(start, start + n, dtype=torch.int64, device=device)
    return _zipf_at(_ZipfRI(n_rows, s), key, pos)


def zipf_pmf(n_rows: int, s: float, k: Sequence[int]) -> List[float]:
    """Exact probabilities of the given ranks (for generator tests)."""
    norm = math.fsum(i ** (-s) for i in range(1, n_rows + 1))
    return [kk ** (-s) / norm for kk in k]


# --------------------------------------------------------------------------------------
# Rank -> row id: seeded bijection on [0, n_rows) (Feistel network + cycle walking)
# --------------------------------------------------------------------------------------
def permute_rows(x: torch.Tensor, n_rows: int, key: int) -> torch.Tensor:
    """Bijection on [0, n_rows): a 4-round balanced Feistel network over the
    smallest even-width power-of-two domain, re-applied while the value falls
    outside the range (cycle walking).  O(1) memory for any table size."""
    assert n_rows >= 1
    if n_rows == 1:
        return torch.zeros_like(x)
    bits = max(2, (n_rows - 1).bit_length())
    hb = (bits + 1) // 2
    mask = (1 << hb) - 1
    rkeys = [mix64_int(key ^ ((r + 1) * 0xA24BAED4963EE407 & _M64)) for r in range(4)]

    def once(v: torch.Tensor) -> torch.Tensor:
        left, right = (v >> hb) & mask, v & mask
        for rk in rkeys:
            f = _lsr(mix64(right * _MULC + _s64(rk)), 64 - hb)
            left, right = right, left ^ f
        return (left << hb) | right

    out = once(x)
    bad = out >= n_rows
    while bool(bad.any()):
        out = torch.where(bad, once(out), out)
        bad = out >= n_rows
    return out


# --------------------------------------------------------------------------------------
# Bag lengths, gradients, weights
# --------------------------------------------------------------------------------------
def _poisson_cdf(lam: float, kmax: int) -> List[float]:
    p, acc, out = math.exp(-lam), 0.0, []
    for k in range(kmax + 1):
        acc += p
        out.append(acc)
        p *= lam / (k + 1)
    return out


def bag_lengths(kind: str, n: int, key: int, start: int = 0,
                device: str | torch.device = "cpu") -> Optional[torch.Tensor]:
    """Per-sample bag lengths.  kinds: ``one`` (None: fixed length 1),
    ``uniform:a:b`` (integers a..b), ``poisson:lam:a:b`` (Poisson clipped to [a,b])."""
    if kind == "one":
        return None
    pos = torch.arange(start, start + n, dtype=torch.int64, device=device)
    u = uniform01(key, pos)
    parts = kind.split(":")
    if parts[0] == "uniform":
        a, b = int(parts[1]), int(parts[2])
        return (a + torch.floor(u * (b - a + 1)).to(torch.int64)).clamp_(a, b)
    if parts[0] == "poisson":
        lam, a, b = float(parts[1]), int(parts[2]), int(parts[3])
        cdf = torch.tensor(_poisson_cdf(lam, max(b, 256)), dtype=torch.float64, device=device)
        k = torch.searchsorted(cdf, u, right=True)
        return k.clamp_(a, b).to(torch.int64)
    raise ValueError(kind)


def normal_f32(shape: Sequence[int], key: int, device: str | torch.device = "cpu") -> torch.Tensor:
    """N(0,1) as fp32 via Box-Muller on two counter-based uniforms (upstream gradients)."""
    n = int(math.prod(shape))
    pos = torch.arange(n, dtype=torch.int64, device=device)
    u1 = uniform01(key, pos * 2)
    u2 = uniform01(key, pos * 2 + 1)
    r = torch.sqrt(-2.0 * torch.log1p(-u1))  # 1-u1 in (0,1]
    return (r * torch.cos(2.0 * math.pi * u2)).to(torch.float32).reshape(*shape)


def w0_key(seed: int, table: int) -> int:
    """Per-table key of the procedural initial weights."""
    return mix64_int(seed ^ ((0x9E3779B97F4A7C15 * (table + 1)) & _M64))


def w0_rows(seed: int, table: int, rows: torch.Tensor, dim: int) -> torch.Tensor:
    """Procedural initial weights U(-0.05, 0.05) of the given rows of a (virtual) table.

    ``h = mix64(key_table + 0xD1B54A32D192ED03 * (row*dim + col + 1))``; the top 24
    bits ``u24`` give ``w = (float(u24) * 2^-24 - 0.5) * 0.1`` in fp32.  Every step
    is exact except the final multiply, which is one correctly rounded fp32
    product, so any IEEE implementation yields the same bits.
    """
    rows = rows.to(torch.int64)
    cols = torch.arange(dim, dtype=torch.int64, device=rows.device)
    ctr = rows[:, None] * dim + cols[None, :] + 1
    h = mix64(ctr * _MULC + _s64(w0_key(seed, table)))
    u24 = _lsr(h, 40).to(torch.float32)
    return (u24 * (2.0 ** -24) - 0.5) * torch.tensor(0.1, dtype=torch.float32, device=rows.device)


# --------------------------------------------------------------------------------------
# Workload configurations
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    rows: tuple            # R_z per table
    dim: int
    bag_kinds: tuple       # per table: "one" | "uniform:a:b" | "poisson:lam:a:b"
    zipf_s: float
    batch: int             # hot-only mini-batch size
    profile_samples: int   # length of the profiled (sampled) stream
    hot_rule: str          # "cutoff" (explicit count) | "budget"
    cutoff: int = 0
    budget_bytes: int = 0
    small_table_bytes: int = 1 << 20
    lr: float = 0.01
    seed: int = SEED
    weights: str = "procedural"
    conditional_hot: bool = False   # hot batches drawn conditionally on the hot set

    @property
    def n_tables(self) -> int:
        return len(self.rows)

    def fixed_len(self, z: int) -> int:
        return 1 if self.bag_kinds[z] == "one" else 0


def loguniform_rows(n_tables: int, lo: float, hi: float, seed: int, cfg_id: int, draw: int) -> tuple:
    """Table cardinalities, log-uniform in [lo, hi].  ``draw`` selects the sub-stream; the
    workloads fix one whose total is close to the expectation of the law, so that the
    hot-row budget actually binds."""
    key = stream_key(seed, cfg_id, draw)
    u = uniform01(key, torch.arange(n_tables, dtype=torch.int64))
    e = math.log10(lo) + u * (math.log10(hi) - math.log10(lo))
    return tuple(int(v) for v in torch.floor(torch.pow(10.0, e)).clamp_(lo, hi).to(torch.int64))


def workload(cfg_id: int, scale: str = "full") -> Workload:
    """The five workloads.  ``scale='test'`` shrinks rows, batch and budget so the CPU
    oracle finishes in seconds while keeping structure (table mix, bag shapes, skew)."""
    full = scale == "full"
    if cfg_id == 1:
        return Workload("cfg1-smoke-1x100k-d16", 1, (100_000,), 16, ("one",), 1.05, 1024,
                        64 * 1024, "cutoff", cutoff=4)
    if cfg_id == 2:
        rows = loguniform_rows(26, 10, 10_000_000 if full else 200_000, SEED, 2, 9001)
        return Workload("cfg2-kaggle-like-26xd16", 2, rows, 16, ("one",) * 26, 1.1,
                        4096 if full else 512, 100_000 if full else 20_000, "budget",
                        budget_bytes=(512 << 20) if full else (8 << 20))
    if cfg_id == 3:
        rows = loguniform_rows(26, 10, 40_000_000 if full else 300_000, SEED, 3, 9002)
        return Workload("cfg3-terabyte-like-26xd64", 3, rows, 64, ("one",) * 26, 1.2,
                        16384 if full else 1024, 1_000_000 if full else 30_000, "budget",
                        budget_bytes=(16 << 30) if full else (48 << 20))
    if cfg_id == 4:
        rows = (1_000_000, 4_000_000, 10_000) if full else (50_000, 200_000, 10_000)
        return Workload("cfg4-taobao-like-3xd32-multihot", 4, rows, 32,
                        ("one", "uniform:1:100", "uniform:1:100"), 1.0,
                        2048 if full else 256, 64 * 2048 if full else 8 * 256, "budget",
                        budget_bytes=(4 << 30) if full else (1 << 30), conditional_hot=True)
    if cfg_id == 5:
        rows = (100_000_000,) * 8 if full else (400_000,) * 8
        return Workload("cfg5-8x100M-d128-poisson20", 5, rows, 128,
                        ("poisson:20:1:64",) * 8, 0.9,
                        65536 if full else 512, (1 << 22) if full else 4096, "budget",
                        budget_bytes=(64 << 30) if full else (256 << 20), conditional_hot=True)
    raise ValueError(cfg_id)


# --------------------------------------------------------------------------------------
# Chunks of the sparse-input stream (CSR per table, table-major)
# --------------------------------------------------------------------------------------
@dataclass
class Chunk:
    n_samples: int
    indices: List[torch.Tensor]             # per table int32[NL_z] (global row ids)
    offsets: List[Optional[torch.Tensor]]   # per table int32[S+1] or None (fixed length 1)
    n_lookups: List[int] = field(default_factory=list)


def _lengths_to_offsets(lens: torch.Tensor) -> torch.Tensor:
    off = torch.zeros(lens.numel() + 1, dtype=torch.int64, device=lens.device)
    torch.cumsum(lens, 0, out=off[1:])
    return off


def make_chunk(w: Workload, stream: int, first_sample: int, n_samples: int,
               device: str | torch.device = "cpu",
               hot_remap: Optional[List[torch.Tensor]] = None) -> Chunk:
    """``n_samples`` consecutive samples of stream ``stream`` starting at ``first_sample``.

    With ``hot_remap`` (per table int32[R_z], negative = cold; passed in as data) every
    lookup is drawn from the Zipf law *conditioned on the hot set*: lookups that hit
    a cold row are redrawn with fresh counters until they hit a hot one.  This is how
    hot-only batches are produced for multi-hot workloads, where an unconditioned
    sample is essentially never all-hot (Sec. 3, challenge 1: the all-hot probability
    decays geometrically with the number of accesses).
    """
    idx_l, off_l, nl_l = [], [], []
    # up to 2^26 lookup slots per sample position keeps streams of different samples disjoint
    for z in range(w.n_tables):
        klen = stream_key(w.seed, w.cfg_id, stream, z, 1)
        kidx = stream_key(w.seed, w.cfg_id, stream, z, 2)
        kperm = stream_key(w.seed, w.cfg_id, z, 3)     # the permutation is per table, not per stream
        lens = bag_lengths(w.bag_kinds[z], n_samples, klen, first_sample, device)
        if lens is None:
            off = None
            pos = torch.arange(first_sample, first_sample + n_samples, dtype=torch.int64, device=device) * 128
        else:
            off = _lengths_to_offsets(lens)
            # stream position of lookup j of sample s = s*128 + j  (bag lengths <= 128)
            sample_of = torch.repeat_interleave(
                torch.arange(first_sample, first_sample + n_samples, dtype=torch.int64, device=device), lens)
            within = torch.arange(int(off[-1]), dtype=torch.int64, device=device) - off[:-1].repeat_interleave(lens)
            pos = sample_of * 128 + within
        nl = pos.numel()
        rows = _draw_rows(w, z, pos, kidx, kperm, device)
        if hot_remap is not None and nl > 0:
            rm = hot_remap[z]
            redo = torch.nonzero(rm[rows] < 0).flatten()
            attempt = 1
            while redo.numel() > 0:
                k2 = stream_key(w.seed, w.cfg_id, stream, z, 2, attempt)
                r2 = _draw_rows(w, z, pos[redo], k2, kperm, device)
                rows[redo] = r2
                redo = redo[rm[r2] < 0]
                attempt += 1
                if attempt > 4096:
                    raise RuntimeError("hot set of table %d looks empty" % z)
        idx_l.append(rows.to(torch.int32))
        off_l.append(None if off is None else off.to(torch.int32))
        nl_l.append(nl)
    return Chunk(n_samples, idx_l, off_l, nl_l)


def _draw_rows(w: Workload, z: int, pos: torch.Tensor, kidx: int, kperm: int, device) -> torch.Tensor:
    if pos.numel() == 0:
        return torch.empty(0, dtype=torch.int64, device=device)
    ranks = _zipf_at(_ZipfRI(w.rows[z], w.zipf_s), kidx, pos)
    return permute_rows(ranks - 1, w.rows[z], kperm)


def sample_chunks(w: "Workload", z: int, m: int, n: int, draw: int = 0) -> List[int]:
    """n distinct chunk numbers out of the ceil(rows_z / m) aligned chunks of table z's
    logger (all of them if there are fewer than n): the first n values of a keyed
    bijection.  Inputs of the sampled hot-size estimate; no arithmetic of the method."""
    N = -(-w.rows[z] // m)
    k = min(n, N)
    key = stream_key(w.seed, 7001, draw, z)
    return [int(v) for v in permute_rows(torch.arange(k, dtype=torch.int64), N, key).tolist()]


def upstream_grads(w: Workload, stream: int, n_samples: int, device: str | torch.device = "cpu") -> torch.Tensor:
    """N(0,1) gradient of the loss w.r.t. the pooled outputs, fp32[S][Tn][dim]."""
    return normal_f32((n_samples, w.n_tables, w.dim), stream_key(w.seed, w.cfg_id, stream, 7), device)


def full_table(w: Workload, z: int, device: str | torch.device = "cpu") -> torch.Tensor:
    """Materialise table z (only sensible at test scale)."""
    return w0_rows(w.seed, z, torch.arange(w.rows[z], dtype=torch.int64, device=device), w.dim)
