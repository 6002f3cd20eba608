"""Shared helpers of the GPU parity tests: run one workload through the HIP library
(C ABI via the binding) and through the CPU oracle on the same seeded inputs and
compare stage by stage.

Tolerances.  Integer outputs (counts, cutoffs, remap, hot ids, sample lists, slots,
offsets, distinct-slot lists, multiplicities) are compared bit-exactly.  fp32
outputs must satisfy |gpu - ref| <= 1e-5 * sum|terms|, where ref is the oracle's
fp64-accumulated result rounded once and the terms are the addends of the sum
(pooled rows; |w_old| and lr*|g_j| for the update): "1e-5 relative" made well
defined under cancellation.  Rows the step does not touch must be bit-identical.
Once a row has been updated its two copies (library, oracle) may differ by that step's
bound; later checks that read the row (the next update, a forward) widen their bound
by exactly that inherited amount (`wtol`), nothing more.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from oracle import fae_oracle as O
from paper_2103_00686_amd import binding as B
from paper_2103_00686_amd import synth as S
from paper_2103_00686_amd.hotpath import HotBatch, HotPath

RTOL = 1e-5


def to_dev(chunk: S.Chunk, dev) -> B.Batch:
    return B.Batch(chunk.n_samples, [i.to(dev) for i in chunk.indices],
                   [None if o is None else o.to(dev) for o in chunk.offsets], list(chunk.n_lookups))


def np_idx(chunk: S.Chunk):
    return ([i.cpu().numpy() for i in chunk.indices],
            [None if o is None else o.cpu().numpy() for o in chunk.offsets])


def assert_close_sum(gpu: np.ndarray, ref: np.ndarray, mag: np.ndarray, what: str, extra=0.0):
    err = np.abs(gpu.astype(np.float64) - ref.astype(np.float64))
    bound = RTOL * mag + extra + 1e-30
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} elements outside 1e-5*sum|terms| " \
                          f"(worst ratio {float((err / bound).max()):.3g})"


def oracle_profile(w: S.Workload, chunks: List[S.Chunk]):
    cnts = [np.zeros(r, dtype=np.uint32) for r in w.rows]
    for ch in chunks:
        idx, _ = np_idx(ch)
        for z in range(w.n_tables):
            O.histogram(w.rows[z], idx[z], cnts[z])
    return cnts


def oracle_hot_rule(w: S.Workload, cnts, chunks):
    """(cutoff[z], n_hot[z], c or None) by the workload's rule."""
    if w.hot_rule == "cutoff":
        H = [w.cutoff] * w.n_tables
        return H, [O.count_hot(c, w.cutoff) for c in cnts], None
    T = [sum(ch.n_lookups[z] for ch in chunks) for z in range(w.n_tables)]
    t_denom = max(max(T), 1)     # one step of c = one access for the most-accessed table
    c, H, nh = O.budget_cutoff(w.dim, cnts, T, t_denom, w.budget_bytes, w.small_table_bytes)
    return [int(h) for h in H], [int(n) for n in nh], c


class Pipeline:
    """Both sides of one workload, kept in step."""

    def __init__(self, w: S.Workload, dev, profile_chunks: int = 2, materialise: bool = False):
        self.w, self.dev = w, dev
        self.hp = HotPath(w.rows, w.dim, dev.index or 0)
        per = -(-w.profile_samples // profile_chunks)
        self.prof = [S.make_chunk(w, 0, i * per, min(per, w.profile_samples - i * per))
                     for i in range(profile_chunks) if i * per < w.profile_samples]
        self.materialise = materialise

    # a1
    def check_profile(self):
        for ch in self.prof:
            self.hp.profile(to_dev(ch, self.dev))
        self.hp.sync()
        self.cnts = oracle_profile(self.w, self.prof)
        for z in range(self.w.n_tables):
            got = self.hp.counts[z][:self.w.rows[z]].cpu().numpy().view(np.uint32)
            assert np.array_equal(got, self.cnts[z]), f"histogram of table {z} differs"

    # a2
    def check_cutoff(self):
        w = self.w
        self.H, self.n_hot, c_ref = oracle_hot_rule(w, self.cnts, self.prof)
        if w.hot_rule == "cutoff":
            assert self.hp.count_hot(self.H) == self.n_hot
        else:
            c, H, nh = self.hp.choose_cutoff(w.budget_bytes, w.small_table_bytes)
            assert (c, H, nh) == (c_ref, self.H, self.n_hot), f"cutoff: gpu {(c, H, nh)} vs oracle {(c_ref, self.H, self.n_hot)}"

    # a3 + a4
    def check_build(self):
        w = self.w
        src = [S.full_table(w, z).to(self.dev) for z in range(w.n_tables)] if self.materialise else None
        got = self.hp.build(self.H, self.n_hot, src_W=src, seed=w.seed)
        assert got == self.n_hot
        self.remap, self.hot_ids, self.hotW = [], [], []
        for z in range(w.n_tables):
            remap, hot_ids = O.classify(self.cnts[z], self.H[z])
            self.remap.append(remap)
            self.hot_ids.append(hot_ids)
            if self.materialise:
                ref_w = O.gather_rows(src[z].cpu().numpy(), hot_ids)
            else:
                ref_w = O.w0_rows(w.seed, z, hot_ids.astype(np.int64), w.dim)
            self.hotW.append(ref_w)
            n = self.n_hot[z]
            if z == 0:
                self.wtol = []
            self.wtol.append(np.zeros(ref_w.shape, dtype=np.float32))   # inherited per-row bound
            assert np.array_equal(self.hp.remap[z][:w.rows[z]].cpu().numpy(), remap), f"remap of table {z} differs"
            assert np.array_equal(self.hp.hot_ids[z][:n].cpu().numpy(), hot_ids), f"hot ids of table {z} differ"
            assert self.hp.hotW[z][:n].cpu().numpy().tobytes() == ref_w.tobytes(), f"hot weights of table {z} differ"

    # a5
    def check_partition(self, chunk: S.Chunk) -> HotBatch:
        w = self.w
        idx, off = np_idx(chunk)
        hs, cs, slots, hoff = O.partition(w.rows, chunk.n_samples, idx, off, self.remap)
        ghs, gcs, hb = self.hp.partition(to_dev(chunk, self.dev))
        assert np.array_equal(ghs.cpu().numpy(), hs), "hot sample list differs"
        assert np.array_equal(gcs.cpu().numpy(), cs), "cold sample list differs"
        assert hb.n_samples == hs.size
        for z in range(w.n_tables):
            assert hb.n_lookups[z] == slots[z].size
            assert np.array_equal(hb.slots[z].cpu().numpy(), slots[z]), f"slots of table {z} differ"
            assert np.array_equal(self.hp.last_hoffsets[z].cpu().numpy(), hoff[z]), f"offsets of table {z} differ"
        return hb

    # a6
    def check_forward(self, hb: HotBatch, exact_gather: bool = True, fused: bool = False):
        """exact_gather: single-row bags must be bit-identical copies (only while the two
        sides hold bit-identical weights, i.e. before the first update).  fused: through
        fae_embbag_fwd_presort (forward and the backward's sort in one launch)."""
        out = (self.hp.forward_presort(hb) if fused else self.hp.forward(hb)).cpu().numpy()
        slots = [s.cpu().numpy() for s in hb.slots]
        offs = [None if o is None else o.cpu().numpy() for o in hb.offsets]
        ref, mag = O.embbag_fwd(self.hotW, hb.n_samples, slots, offs, want_mag=True)
        inherited = O.embbag_fwd(self.wtol, hb.n_samples, slots, offs).astype(np.float64) * 1.001
        assert_close_sum(out, ref, mag, "forward", inherited)
        for z, o in enumerate(offs):   # single-row bags involve no arithmetic: bit-exact
            if hb.n_samples == 0 or not exact_gather:
                continue
            if o is None:
                assert out[:, z, :].tobytes() == ref[:, z, :].tobytes(), f"one-hot table {z} is not a bit-exact gather"
            else:
                one = np.diff(o) <= 1
                assert out[one, z, :].tobytes() == ref[one, z, :].tobytes()
        return out

    # a7 + a8
    def check_backward(self, hb: HotBatch, stream: int, presort: Optional[HotBatch] = None):
        """presort: start the backward's sort for that batch on the side stream first (the same
        batch: the sorted pairs are reused; another batch: they must be ignored)."""
        w = self.w
        if presort is not None:
            self.hp.presort(presort)
        gout = S.upstream_grads(w, stream, hb.n_samples)
        before = [x.clone() for x in self.hp.hotW]      # device-side snapshot of the library's own state
        dbg = self.hp.backward_sgd(hb, gout.to(self.dev), w.lr, debug=True)
        self.hp.sync()
        slots = [s.cpu().numpy() for s in hb.slots]
        offs = [None if o is None else o.cpu().numpy() for o in hb.offsets]
        uniq, runlen, mag = O.embbag_bwd_sgd(self.hotW, hb.n_samples, slots, offs, gout.numpy(), w.lr, want_mag=True)
        for z in range(w.n_tables):
            assert np.array_equal(dbg[0][z].cpu().numpy(), uniq[z]), f"distinct slots of table {z} differ"
            assert np.array_equal(dbg[1][z].cpu().numpy(), runlen[z]), f"multiplicities of table {z} differ"
            got = self.hp.hotW[z][:self.n_hot[z]].cpu().numpy()
            touched = np.zeros(self.n_hot[z], dtype=bool)
            touched[uniq[z]] = True
            prev = before[z][:self.n_hot[z]].cpu().numpy()
            assert got[~touched].tobytes() == prev[~touched].tobytes(), f"untouched rows of table {z} changed"
            if uniq[z].size:
                inherited = self.wtol[z][uniq[z]].astype(np.float64)
                assert_close_sum(got[uniq[z]], self.hotW[z][uniq[z]], mag[z], f"updated rows of table {z}", inherited)
                self.wtol[z][uniq[z]] = (inherited + RTOL * mag[z]).astype(np.float32) * np.float32(1.001)


    def check_step(self, hb: HotBatch, out: torch.Tensor, gout: torch.Tensor):
        """After the library has run forward and backward/SGD of hb on its own (any call pattern):
        the pooled output against the oracle's forward with the weights before the step, then the
        updated rows against the oracle's update (which also advances the oracle's weights)."""
        w = self.w
        slots = [s.cpu().numpy() for s in hb.slots]
        offs = [None if o is None else o.cpu().numpy() for o in hb.offsets]
        ref, mag = O.embbag_fwd(self.hotW, hb.n_samples, slots, offs, want_mag=True)
        inherited = O.embbag_fwd(self.wtol, hb.n_samples, slots, offs).astype(np.float64) * 1.001
        assert_close_sum(out.cpu().numpy(), ref, mag, "forward", inherited)
        uniq, runlen, mg = O.embbag_bwd_sgd(self.hotW, hb.n_samples, slots, offs, gout.cpu().numpy(), w.lr, want_mag=True)
        for z in range(w.n_tables):
            if uniq[z].size:
                got = self.hp.hotW[z][:self.n_hot[z]].cpu().numpy()
                inh = self.wtol[z][uniq[z]].astype(np.float64)
                assert_close_sum(got[uniq[z]], self.hotW[z][uniq[z]], mg[z], f"updated rows of table {z}", inh)
                self.wtol[z][uniq[z]] = (inh + RTOL * mg[z]).astype(np.float32) * np.float32(1.001)


class SparseTables:
    """The oracle's copy of hot tables that are too large to hold on the host: only rows that some
    step has updated are kept (with the error bound they have inherited, see the module header);
    every other row is the procedural initial weight W0(seed, table, row)."""

    def __init__(self, seed: int, hot_ids: List[np.ndarray], dim: int):
        self.seed, self.hot_ids, self.dim = seed, hot_ids, dim
        nt = len(hot_ids)
        self.slots = [np.empty(0, dtype=np.int64) for _ in range(nt)]
        self.rows = [np.empty((0, dim), dtype=np.float32) for _ in range(nt)]
        self.tol = [np.empty((0, dim), dtype=np.float32) for _ in range(nt)]

    def fetch(self, z: int, want: np.ndarray):
        """Current rows (and inherited bounds) of the ascending distinct slots `want` of table z."""
        want = np.asarray(want, dtype=np.int64)
        rows = O.w0_rows(self.seed, z, self.hot_ids[z][want].astype(np.int64), self.dim)
        tol = np.zeros(rows.shape, dtype=np.float32)
        have = self.slots[z]
        if have.size and want.size:
            pos = np.minimum(np.searchsorted(have, want), have.size - 1)
            hit = have[pos] == want
            rows[hit] = self.rows[z][pos[hit]]
            tol[hit] = self.tol[z][pos[hit]]
        return rows, tol

    def store(self, z: int, slots: np.ndarray, rows: np.ndarray, tol: np.ndarray):
        slots = np.asarray(slots, dtype=np.int64)
        keep = ~np.isin(self.slots[z], slots)
        all_slots = np.concatenate([self.slots[z][keep], slots])
        order = np.argsort(all_slots, kind="stable")
        self.slots[z] = all_slots[order]
        self.rows[z] = np.concatenate([self.rows[z][keep], rows])[order]
        self.tol[z] = np.concatenate([self.tol[z][keep], tol])[order]

    def touched(self, z: int) -> np.ndarray:
        return self.slots[z]


def check_step_sparse(store: SparseTables, hp: HotPath, n_samples: int, slots: List[np.ndarray],
                      offs: List[Optional[np.ndarray]], out: torch.Tensor, gout: torch.Tensor, lr: float, what: str,
                      dbg=None):
    """One step that the library has already taken on its own tables (any call sequence), against
    the oracle, table by table and in full: every pooled row against the oracle's forward with the
    weights before the step, every updated row against the oracle's update, and (when the library's
    optional outputs are given) the distinct slots and their multiplicities bit for bit.  The oracle
    works on the rows the batch touches, compacted; its tables advance with the step."""
    dev = out.device
    nt = len(slots)
    for z in range(nt):
        sl = np.asarray(slots[z], dtype=np.int32)
        uniq_slots, inv = np.unique(sl, return_inverse=True)
        inv = inv.astype(np.int32)
        if uniq_slots.size == 0:
            assert not bool(out[:, z, :].any()), f"{what}: table {z} has no lookups but a non-zero output"
            continue
        Wc, tolc = store.fetch(z, uniq_slots)
        ref, mag = O.embbag_fwd([Wc], n_samples, [inv], [offs[z]], want_mag=True)
        inherited = O.embbag_fwd([tolc], n_samples, [inv], [offs[z]]).astype(np.float64) * 1.001
        got = out[:, z, :].cpu().numpy()
        assert_close_sum(got, ref[:, 0, :], mag[:, 0, :], f"{what}: forward, table {z}", inherited[:, 0, :])
        g_z = np.ascontiguousarray(gout[:, z:z + 1, :].cpu().numpy())
        uniq, runlen, mg = O.embbag_bwd_sgd([Wc], n_samples, [inv], [offs[z]], g_z, lr, want_mag=True)
        assert np.array_equal(uniq[0], np.arange(uniq_slots.size))      # every compacted row is touched
        if dbg is not None:
            assert np.array_equal(dbg[0][z].cpu().numpy(), uniq_slots), f"{what}: distinct slots of table {z} differ"
            assert np.array_equal(dbg[1][z].cpu().numpy(), runlen[0]), f"{what}: multiplicities of table {z} differ"
        got_rows = hp.hotW[z][torch.from_numpy(uniq_slots.astype(np.int64)).to(dev)].cpu().numpy()
        assert_close_sum(got_rows, Wc, mg[0], f"{what}: updated rows, table {z}", tolc.astype(np.float64))
        newtol = (tolc.astype(np.float64) + RTOL * mg[0]).astype(np.float32) * np.float32(1.001)
        store.store(z, uniq_slots, Wc, newtol)


def hot_batches(p: Pipeline, n_batches: int, stream0: int = 10) -> List[HotBatch]:
    """Hot-only mini-batches of the workload's batch size, the way the workload makes them:
    conditional-hot draws for multi-hot workloads, partition of a mixed stream otherwise."""
    w = p.w
    out = []
    if w.conditional_hot:
        remap_t = [torch.from_numpy(r) for r in p.remap]
        for b in range(n_batches):
            ch = S.make_chunk(w, stream0 + b, 0, w.batch, hot_remap=remap_t)
            hb = p.check_partition(ch)
            assert hb.n_samples == w.batch
            out.append(hb)
        return out
    need, first, got = n_batches * w.batch, 0, []
    hb_all: Optional[HotBatch] = None
    span = max(4 * need, 4096)
    ch = S.make_chunk(w, stream0, first, span)
    hb_all = p.check_partition(ch)
    n_full = hb_all.n_samples // w.batch
    for b in range(min(n_batches, n_full)):
        out.append(hb_all.slice(b * w.batch, w.batch))
    if not out:      # very selective hot set: use whatever is hot as one ragged batch
        out.append(hb_all)
    return out
