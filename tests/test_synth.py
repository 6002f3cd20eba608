"""The seeded input generators: exact Zipf law, bijective row permutation, position-only
dependence (chunking does not change the stream), conditional-hot draws."""
import math

import numpy as np
import torch

from paper_2103_00686_amd import synth as S


def test_zipf_matches_exact_pmf():
    n, R, s = 400_000, 500, 1.1
    r = S.zipf_ranks(n, R, s, S.stream_key(1, 2))
    assert int(r.min()) >= 1 and int(r.max()) <= R
    ks = [1, 2, 3, 7, 50, 500]
    for k, p in zip(ks, S.zipf_pmf(R, s, ks)):
        f = float((r == k).double().mean())
        assert abs(f - p) < 5 * math.sqrt(p * (1 - p) / n) + 1e-6
    # s = 1 (log form) and s < 1
    for s in (1.0, 0.9):
        r = S.zipf_ranks(200_000, 100, s, 5)
        p1, = S.zipf_pmf(100, s, [1])
        assert abs(float((r == 1).double().mean()) - p1) < 5 * math.sqrt(p1 / 200_000)


def test_permutation_is_a_bijection():
    for R in (1, 2, 3, 10, 1000, 4097, 65536):
        y = S.permute_rows(torch.arange(R), R, 99)
        assert sorted(y.tolist()) == list(range(R))


def test_stream_is_position_addressed():
    w = S.workload(4, "test")
    a = S.make_chunk(w, 3, 0, 64)
    b = S.make_chunk(w, 3, 32, 32)
    for z in range(w.n_tables):
        if a.offsets[z] is None:
            assert a.indices[z][32:].tolist() == b.indices[z].tolist()
        else:
            cut = int(a.offsets[z][32])
            assert a.indices[z][cut:].tolist() == b.indices[z].tolist()
            assert (a.offsets[z][32:] - cut).tolist() == b.offsets[z].tolist()


def test_workload_shapes():
    for cid in range(1, 6):
        for scale in ("full", "test"):
            w = S.workload(cid, scale)
            assert len(w.bag_kinds) == w.n_tables
    w = S.workload(5, "test")
    c = S.make_chunk(w, 0, 0, 2000)
    lens = torch.diff(c.offsets[0])
    assert int(lens.min()) >= 1 and int(lens.max()) <= 64 and abs(float(lens.double().mean()) - 20) < 0.5
    for z in range(w.n_tables):
        assert c.indices[z].dtype == torch.int32 and int(c.indices[z].max()) < w.rows[z]
        assert c.n_lookups[z] == c.indices[z].numel() == int(c.offsets[z][-1])


def test_conditional_hot_draws_only_hot_rows():
    w = S.workload(5, "test")
    remap = []
    for z in range(w.n_tables):
        r = torch.full((w.rows[z],), -1, dtype=torch.int32)
        hot = S.permute_rows(torch.arange(2000), w.rows[z], S.stream_key(w.seed, w.cfg_id, z, 3))
        r[hot] = 1
        remap.append(r)
    c = S.make_chunk(w, 1, 0, 100, hot_remap=remap)
    free = S.make_chunk(w, 1, 0, 100)
    for z in range(w.n_tables):
        assert bool((remap[z][c.indices[z].long()] >= 0).all())
        assert c.offsets[z].tolist() == free.offsets[z].tolist()
        keep = remap[z][free.indices[z].long()] >= 0           # already-hot draws are kept
        assert c.indices[z][keep].tolist() == free.indices[z][keep].tolist()


def test_grads_are_standard_normal():
    g = S.upstream_grads(S.workload(1), 0, 4096)
    assert g.shape == (4096, 1, 16) and g.dtype == torch.float32
    assert abs(float(g.mean())) < 0.02 and abs(float(g.std()) - 1) < 0.02
