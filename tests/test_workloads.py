"""The seeded input generators: shapes, ranges, determinism and the stated degree laws."""
import numpy as np

from paper_2502_16949_amd import workloads as W


def test_graph_shapes_and_determinism():
    wl = W.WORKLOADS["mid"]
    h, r, t = W.make_graph(wl)
    h2, r2, t2 = W.make_graph(wl)
    assert all(np.array_equal(a, b) for a, b in ((h, h2), (r, r2), (t, t2)))
    assert h.dtype == np.int32 and len(h) == len(r) == len(t) == 480_000
    assert 0 <= h.min() and h.max() < wl.n_ent and 0 <= t.min() and t.max() < wl.n_ent
    assert 0 <= r.min() and r.max() < wl.n_rel
    assert wl.rows_per_batch == 65_536 and wl.n_batches == 15
    assert W.batch_slices(wl)[-1] == (14 * 32_768, 480_000)


def test_zipf_law_matches_exponent():
    wl = W.WORKLOADS["mid"]
    h, r, _ = W.make_graph(wl)
    for ids, n, s in ((h, wl.n_ent, wl.zipf_ent), (r, wl.n_rel, wl.zipf_rel)):
        cnt = np.sort(np.bincount(ids, minlength=n))[::-1].astype(np.float64)
        p1 = 1.0 / np.sum(np.arange(1, n + 1, dtype=np.float64) ** -s)
        assert abs(cnt[0] / len(ids) - p1) < 0.01                  # mass of the top rank
        slope = np.polyfit(np.log(np.arange(1, 21)), np.log(cnt[:20]), 1)[0]
        assert abs(-slope - s) < 0.15                              # log-log slope over the top 20 ranks


def test_tables():
    for name in ("tiny", "transh", "transr"):
        wl = W.WORKLOADS[name]
        tabs = W.make_tables(wl)
        a = 6 / np.sqrt(wl.dim)
        assert tabs["ent"].dtype == np.float32 and np.abs(tabs["ent"]).max() <= a
        if name == "tiny":
            assert tabs["ent"].shape == (wl.n_ent + wl.n_rel, wl.dim)
        if name == "transh":
            np.testing.assert_allclose(np.linalg.norm(tabs["w"].astype(np.float64), axis=1), 1, atol=1e-6)
        if name == "transr":
            assert tabs["proj"].shape == (wl.n_rel, wl.rel_dim, wl.dim)
            assert abs(tabs["proj"].var() * wl.dim - 1) < 0.02
    small = W.WORKLOADS["toruse"].scaled(n_ent=1000, n_rel=10)
    x = W.make_tables(small)["ent"]
    assert x.min() >= 0 and x.max() < 1
