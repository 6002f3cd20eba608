"""Convenience driver around the C ABI: allocates device buffers and workspaces with
torch (plumbing only) and calls the library stage by stage in the paper's order
(Sec. 4: profile -> cutoff -> classify/replicate -> input classifier -> hot
mini-batch forward / backward / SGD).  No arithmetic of the method happens here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as B


@dataclass
class HotBatch:
    """A hot-only batch over the hot tables (slots instead of row ids)."""
    n_samples: int
    slots: List[torch.Tensor]
    offsets: List[Optional[torch.Tensor]]
    n_lookups: List[int]

    def batch(self) -> B.Batch:
        if getattr(self, "_b", None) is None:
            self._b = B.Batch(self.n_samples, self.slots, self.offsets, self.n_lookups)
        return self._b

    def slice(self, first: int, count: int) -> "HotBatch":
        """Samples [first, first+count) as a batch of their own (offsets rebased to 0)."""
        count = max(0, min(count, self.n_samples - first))
        slots, offs, nl = [], [], []
        for s, o in zip(self.slots, self.offsets):
            if o is None:
                slots.append(s[first:first + count])
                offs.append(None)
                nl.append(count)
            else:
                lo, hi = int(o[first]), int(o[first + count])
                slots.append(s[lo:hi])
                offs.append((o[first:first + count + 1] - lo).contiguous())
                nl.append(hi - lo)
        return HotBatch(count, slots, offs, nl)


class HotPath:
    def __init__(self, rows: Sequence[int], dim: int, device: int = 0, stream: Optional[int] = None):
        """stream: a hipStream_t handle (e.g. ``torch.cuda.Stream().cuda_stream``); default is
        torch's current stream at construction.  Every library call is queued there."""
        self.dev = torch.device("cuda", device)
        self.ctx = B.Context(device, stream)
        self.tables = B.Tables(list(rows), dim)
        self.dim = dim
        self.nt = len(rows)
        self.counts: Optional[List[torch.Tensor]] = None
        self.profiled_lookups = [0] * self.nt
        self.profiled_samples = 0
        self.remap = self.hot_ids = self.hotW = None
        self.n_hot: List[int] = []
        self._ws = {}

    # -- plumbing -----------------------------------------------------------------
    def _workspace(self, name: str, nbytes: int) -> torch.Tensor:
        ws = self._ws.get(name)
        if ws is None or ws.numel() < nbytes:
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.dev)
            self._ws[name] = ws
        return ws

    @property
    def hot_tables(self) -> B.Tables:
        t = getattr(self, "_hot_tables", None)
        if t is None or list(t.rows) != list(self.n_hot):
            t = self._hot_tables = B.Tables(list(self.n_hot), self.dim)
        return t

    def prepare_step(self, hb: HotBatch, gout: torch.Tensor, out: torch.Tensor, lr: float, presort: str = "fused"):
        """Pre-marshalled forward + backward/SGD on one hot batch: returns a zero-argument
        callable that only issues the library calls (for tight training loops).  presort:
        "fused" = forward and the backward's sort in one launch where the shape allows,
        "side" = the sort on the side stream before the forward, "none" = separate calls."""
        import ctypes as C
        lib = B.load()
        t, b = self.hot_tables.c(), hb.batch().c()
        wptr = B._ptrs(self.hotW, torch.float32)
        ws = self.bwd_workspace(hb)
        stride = C.c_int64(self.nt * self.dim)
        a_out, a_gout, a_ws = C.c_void_p(out.data_ptr()), C.c_void_p(gout.data_ptr()), C.c_void_p(ws.data_ptr())
        n_ws, c_lr, h = C.c_size_t(ws.numel()), C.c_float(lr), self.ctx._h
        tr, br = C.byref(t), C.byref(b)
        keep = (t, b, wptr, ws, out, gout, hb)

        def step():
            if presort == "fused":
                rc = lib.fae_embbag_fwd_presort(h, tr, wptr, br, a_out, stride, a_ws, n_ws)
            else:
                rc = lib.fae_embbag_bwd_presort(h, tr, br, a_ws, n_ws) if presort == "side" else 0
                if rc == 0:
                    rc = lib.fae_embbag_fwd(h, tr, wptr, br, a_out, stride)
            if rc == 0:
                rc = lib.fae_embbag_bwd_sgd(h, tr, wptr, br, a_gout, stride, c_lr, None, a_ws, n_ws)
            if rc != 0:
                self.ctx.check(rc)
        step._keep = keep
        return step

    def prepare_pipeline(self, hbs: Sequence[HotBatch], gouts: Sequence[torch.Tensor], outs: Sequence[torch.Tensor],
                         lr: float):
        """Steps over a cycle of hot batches whose backward sorts run one step ahead: step i
        starts the sort of batch i+1 on the side stream (into the other of two workspaces), then
        runs forward and backward/SGD of batch i, whose pairs were sorted during step i-1.  Hot
        mini-batches are formed ahead of training (Sec. 4), so the next batch is always known.
        Returns one zero-argument callable per batch; they must be called in cyclic order."""
        import ctypes as C
        lib = B.load()
        n = len(hbs)
        need = max(B.fae_bwd_workspace_bytes(self.hot_tables, hb.n_samples, hb.n_lookups) for hb in hbs)
        wss = [self._workspace(f"bwd_ahead{i}", need) for i in range(2)]
        a_ws = [C.c_void_p(w.data_ptr()) for w in wss]
        n_ws = [C.c_size_t(w.numel()) for w in wss]
        t = self.hot_tables.c()
        tr = C.byref(t)
        wptr = B._ptrs(self.hotW, torch.float32)
        stride, c_lr, h = C.c_int64(self.nt * self.dim), C.c_float(lr), self.ctx._h
        bs = [hb.batch().c() for hb in hbs]
        brs = [C.byref(b) for b in bs]
        a_out = [C.c_void_p(o.data_ptr()) for o in outs]
        a_gout = [C.c_void_p(g.data_ptr()) for g in gouts]
        state = {"k": 0}
        keep = (t, bs, wptr, wss, outs, gouts, hbs)

        def make(i):
            j = (i + 1) % n

            def step():
                k = state["k"]
                cur, nxt = k & 1, (k + 1) & 1
                rc = lib.fae_embbag_bwd_presort(h, tr, brs[j], a_ws[nxt], n_ws[nxt])
                if rc == 0:
                    rc = lib.fae_embbag_fwd(h, tr, wptr, brs[i], a_out[i], stride)
                if rc == 0:
                    rc = lib.fae_embbag_bwd_sgd(h, tr, wptr, brs[i], a_gout[i], stride, c_lr, None, a_ws[cur], n_ws[cur])
                state["k"] = k + 1
                if rc != 0:
                    self.ctx.check(rc)
            step._keep = keep
            return step
        return [make(i) for i in range(n)]

    def prepare_steps(self, hbs: Sequence[HotBatch], gouts: Sequence[torch.Tensor], outs: Sequence[torch.Tensor],
                      lr: float, presort: str = "auto", single_stream: bool = False):
        """The training steps of a cycle of hot batches as zero-argument callables (to be called in
        cyclic order), and the name of the call sequence they use.  presort "auto" picks, from the
        shapes alone: "fused" (forward and the backward's sort in one launch) when every table is
        one-hot and the batches have at most 16384 samples; "ahead" (the next batch's sort on the
        side stream beside this batch's forward and backward) for other steps of up to 4 M lookups,
        whose sort is a string of short launches; else the calls one after the other ("fused", which
        is the plain forward for such shapes).  single_stream rules "ahead" out (graph capture)."""
        if presort == "auto":
            fusable = all(o is None for hb in hbs for o in hb.offsets) and max(hb.n_samples for hb in hbs) <= 16384
            short_sort = max(sum(hb.n_lookups) for hb in hbs) <= (1 << 22)
            presort = "ahead" if (not fusable and short_sort and not single_stream) else "fused"
        if presort == "ahead":
            return self.prepare_pipeline(hbs, gouts, outs, lr), presort
        return [self.prepare_step(hb, g, o, lr, presort=presort) for hb, g, o in zip(hbs, gouts, outs)], presort

    # -- a1 -------------------------------------------------------------------------
    def alloc_counts(self):
        """Access counters of every table, zeroed (profile() makes them on first use otherwise)."""
        self.counts = [torch.zeros(max(int(r), 1), dtype=torch.int32, device=self.dev) for r in self.tables.rows]
        self.profiled_samples = 0
        self.profiled_lookups = [0] * self.nt

    def profile(self, chunk: B.Batch):
        if self.counts is None:
            self.alloc_counts()
        B.fae_profile(self.ctx, self.tables, chunk, self.counts)
        self.profiled_samples += chunk.n_samples
        for z in range(self.nt):
            self.profiled_lookups[z] += int(chunk.n_lookups[z])

    # -- a2 -------------------------------------------------------------------------
    def choose_cutoff(self, budget_bytes: int, small_table_bytes: int = 1 << 20):
        ws = self._workspace("cut", B.fae_choose_cutoff_workspace_bytes(self.tables))
        # threshold grid: one step of c = one access for the most-accessed table
        return B.fae_choose_cutoff(self.ctx, self.tables, self.counts, self.profiled_lookups,
                                   max(max(self.profiled_lookups), 1), budget_bytes, small_table_bytes, ws)

    def count_hot(self, cutoff: Sequence[int]) -> List[int]:
        ws = self._workspace("cut", B.fae_choose_cutoff_workspace_bytes(self.tables))
        return B.fae_count_hot(self.ctx, self.tables, self.counts, cutoff, ws)

    # -- sampled estimate of the hot size (Sec. 4.1.2, Eq. 2-4) ----------------------
    def estimate_hot(self, cutoff: Sequence[int], chunks: Sequence[Sequence[int]], m: int = 1024,
                     confidence: float = 0.999):
        ws = self._workspace("est", B.fae_estimate_workspace_bytes(self.tables, [len(c) for c in chunks]))
        return B.fae_estimate_hot(self.ctx, self.tables, self.counts, cutoff, m, chunks, confidence, ws)

    def choose_cutoff_sampled(self, budget_bytes: int, chunks: Sequence[Sequence[int]], m: int = 1024,
                              confidence: float = 0.999, small_table_bytes: int = 1 << 20):
        ws = self._workspace("est", B.fae_estimate_workspace_bytes(self.tables, [len(c) for c in chunks]))
        return B.fae_choose_cutoff_sampled(self.ctx, self.tables, self.counts, self.profiled_lookups,
                                           max(max(self.profiled_lookups), 1), budget_bytes, small_table_bytes,
                                           m, chunks, confidence, ws)

    # -- hot <-> full table synchronisation (Sec. 3 (4), Sec. 6.2) -----------------------
    def sync_to_full(self, W: List[torch.Tensor]):
        B.fae_sync_hot_rows(self.ctx, self.tables, self.n_hot, self.hot_ids, self.hotW, W, B.FAE_SYNC_HOT_TO_FULL)

    def sync_from_full(self, W: List[torch.Tensor]):
        B.fae_sync_hot_rows(self.ctx, self.tables, self.n_hot, self.hot_ids, self.hotW, W, B.FAE_SYNC_FULL_TO_HOT)

    # -- a3 + a4 --------------------------------------------------------------------
    def build(self, cutoff: Sequence[int], n_hot: Sequence[int], src_W: Optional[List[torch.Tensor]] = None,
              seed: int = 0) -> List[int]:
        self.remap = [torch.empty(max(int(r), 1), dtype=torch.int32, device=self.dev) for r in self.tables.rows]
        self.hot_ids = [torch.empty(max(int(n), 1), dtype=torch.int32, device=self.dev) for n in n_hot]
        self.hotW = [torch.empty((max(int(n), 1), self.dim), dtype=torch.float32, device=self.dev) for n in n_hot]
        ws = self._workspace("build", B.fae_build_workspace_bytes(self.tables))
        kind = B.FAE_SRC_DEVICE if src_W is not None else B.FAE_SRC_PROCEDURAL
        got = B.fae_build_hot_tables(self.ctx, self.tables, self.counts, cutoff, kind, src_W, seed,
                                     self.remap, self.hot_ids, self.hotW, [int(n) for n in n_hot], ws)
        self.n_hot = [int(n) for n in got]
        return self.n_hot

    # -- a5 -------------------------------------------------------------------------
    def partition(self, batch: B.Batch):
        """Returns (hot_samples, cold_samples, HotBatch)."""
        S = batch.n_samples
        hot = torch.empty(max(S, 1), dtype=torch.int32, device=self.dev)
        cold = torch.empty(max(S, 1), dtype=torch.int32, device=self.dev)
        slots = [torch.empty(max(int(n), 1), dtype=torch.int32, device=self.dev) for n in batch.n_lookups]
        hoff = [torch.empty(S + 1, dtype=torch.int32, device=self.dev) for _ in range(self.nt)]
        ws = self._workspace("part", B.fae_partition_workspace_bytes(self.tables, S))
        n_hot, nl = B.fae_partition_batch(self.ctx, self.tables, batch, self.remap, hot, cold, slots, hoff, ws)
        hb = HotBatch(n_hot,
                      [s[:n] for s, n in zip(slots, nl)],
                      [None if o is None else h[:n_hot + 1] for o, h in zip(batch.offsets, hoff)],
                      [int(n) for n in nl])
        self.last_hoffsets = [h[:n_hot + 1] for h in hoff]
        return hot[:n_hot], cold[:S - n_hot], hb

    # -- a6 -------------------------------------------------------------------------
    def forward(self, hb: HotBatch, out: Optional[torch.Tensor] = None, pooling: int = B.FAE_POOL_SUM) -> torch.Tensor:
        if out is None:
            out = torch.empty((hb.n_samples, self.nt, self.dim), dtype=torch.float32, device=self.dev)
        if pooling == B.FAE_POOL_SUM:
            B.fae_embbag_fwd(self.ctx, self.hot_tables, self.hotW, hb.batch(), out, self.nt * self.dim)
        else:
            B.fae_embbag_fwd_opts(self.ctx, self.hot_tables, self.hotW, hb.batch(), out, self.nt * self.dim, pooling)
        return out

    # -- a7 + a8 --------------------------------------------------------------------
    def bwd_workspace(self, hb: HotBatch) -> torch.Tensor:
        return self._workspace("bwd", B.fae_bwd_workspace_bytes(self.hot_tables, hb.n_samples, hb.n_lookups))

    def presort(self, hb: HotBatch):
        B.fae_embbag_bwd_presort(self.ctx, self.hot_tables, hb.batch(), self.bwd_workspace(hb))

    def forward_presort(self, hb: HotBatch, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty((hb.n_samples, self.nt, self.dim), dtype=torch.float32, device=self.dev)
        B.fae_embbag_fwd_presort(self.ctx, self.hot_tables, self.hotW, hb.batch(), out, self.nt * self.dim,
                                 self.bwd_workspace(hb))
        return out

    def backward_sgd(self, hb: HotBatch, gout: torch.Tensor, lr: float, debug: bool = False):
        ws = self.bwd_workspace(hb)
        if not debug:
            B.fae_embbag_bwd_sgd(self.ctx, self.hot_tables, self.hotW, hb.batch(), gout, self.nt * self.dim, lr, ws)
            return None
        n = max(sum(hb.n_lookups), 1)
        uniq = torch.empty(n, dtype=torch.int32, device=self.dev)
        runlen = torch.empty(n, dtype=torch.int32, device=self.dev)
        tstart = torch.zeros(self.nt + 1, dtype=torch.int32, device=self.dev)
        B.fae_embbag_bwd_sgd(self.ctx, self.hot_tables, self.hotW, hb.batch(), gout, self.nt * self.dim, lr, ws,
                             uniq, runlen, tstart)
        ts = tstart.cpu().tolist()
        return ([uniq[ts[z]:ts[z + 1]] for z in range(self.nt)], [runlen[ts[z]:ts[z + 1]] for z in range(self.nt)])

    def backward_opts(self, hb: HotBatch, gout: torch.Tensor, lr: float, pooling: int = B.FAE_POOL_SUM,
                      optimizer: int = B.FAE_OPT_SGD, eps: float = 0.0, state: Optional[List[torch.Tensor]] = None):
        """Backward with a pooling / optimizer variant; returns the distinct slots and their
        multiplicities per table like ``backward_sgd(debug=True)``."""
        ws = self.bwd_workspace(hb)
        n = max(sum(hb.n_lookups), 1)
        uniq = torch.empty(n, dtype=torch.int32, device=self.dev)
        runlen = torch.empty(n, dtype=torch.int32, device=self.dev)
        tstart = torch.zeros(self.nt + 1, dtype=torch.int32, device=self.dev)
        B.fae_embbag_bwd_opts(self.ctx, self.hot_tables, self.hotW, hb.batch(), gout, self.nt * self.dim, lr, ws,
                              pooling, optimizer, eps, state, uniq, runlen, tstart)
        ts = tstart.cpu().tolist()
        return ([uniq[ts[z]:ts[z + 1]] for z in range(self.nt)], [runlen[ts[z]:ts[z + 1]] for z in range(self.nt)])

    def sync(self):
        B.fae_sync(self.ctx)
