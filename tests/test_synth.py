"""The seeded input generators: sorted, distinct, reproducible, of the requested size and skew."""
import numpy as np

from paper_2311_09549_amd import synth


def _keys(coords, dims):
    key = np.zeros(coords.shape[1], dtype=np.int64)
    for m in range(coords.shape[0]):
        key = key * int(dims[m]) + coords[m]
    return key


def test_sorted_distinct_exact_nnz_all_configs_shrunk():
    for cid, scale in [(1, 1.0), (2, 0.002), (3, 0.002), (4, 0.002), (5, 0.01)]:
        cfg = synth.config(cid, scale)
        d = synth.generate(cfg)
        c = d["coords"]
        assert c.dtype == np.int32 and c.shape == (len(cfg["dims"]), cfg["nnz"])
        for m, dim in enumerate(cfg["dims"]):
            assert c[m].min() >= 0 and c[m].max() < dim
        assert np.all(np.diff(_keys(c, cfg["dims"])) > 0)  # strictly increasing: sorted and distinct
        assert d["vals"].shape == (cfg["nnz"],) and np.abs(d["vals"]).max() <= 1.0
        for f, shp in zip(d["factors"], synth.factor_shapes(cfg)):
            assert f.shape == shp and f.flags.c_contiguous


def test_reproducible_and_seed_dependent():
    cfg = synth.config(2, 0.001)
    a, b = synth.generate(cfg), synth.generate(cfg)
    assert np.array_equal(a["coords"], b["coords"]) and np.array_equal(a["vals"], b["vals"])
    cfg2 = dict(cfg, seed_offset=1)
    c = synth.generate(cfg2)
    assert not np.array_equal(a["coords"], c["coords"])


def test_zipf_is_skewed_and_uniform_is_not():
    cfg = synth.config(3, 0.01)
    c = synth.generate(cfg)["coords"]
    counts = np.sort(np.bincount(c[0], minlength=cfg["dims"][0]))[::-1]
    assert counts[0] > 20 * np.median(counts[counts > 0])
    cfg1 = synth.config(1)
    c1 = synth.generate(cfg1)["coords"]
    counts1 = np.bincount(c1[0], minlength=200)
    assert counts1.max() < 3 * counts1.mean()
