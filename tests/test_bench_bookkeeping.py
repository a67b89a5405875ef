"""bench.py's own density / FLOP bookkeeping against the oracle's and against a brute-force
block count (CPU only: bench.py is imported, not run)."""
import importlib.util
import os
from types import SimpleNamespace

import numpy as np
import pytest

from oracle import s2o_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _w(L, S, BM, BN, Z=1, H=3, D=128):
    return SimpleNamespace(L=L, S=S, N=L // S, BM=BM, BN=BN, Z=Z, H=H, D=D)


@pytest.mark.parametrize("L,S,BM,BN", [(2048, 256, 64, 64), (2048, 512, 128, 64), (8192, 1024, 128, 64),
                                       (131072, 2048, 64, 64), (131072, 2048, 128, 64)])
def test_density_and_flops_agree_with_the_oracle(bench, L, S, BM, BN):
    w = _w(L, S, BM, BN)
    pre = orc.prefix_tiles(L, S, BM, BN)
    assert np.array_equal(bench.prefix_tiles(w), pre)
    rng = np.random.default_rng(L // BM)
    for _ in range(3):
        skipped = rng.integers(0, pre + 1, size=(w.Z, w.H, L // BM))
        trig = rng.integers(0, 2, size=skipped.shape) * (skipped < pre)     # a discarded trigger only if one was issued
        computed = pre[None, None] - skipped - trig
        np.testing.assert_allclose(bench.density_of(w, skipped), orc.density(skipped, L, S, BM, BN), rtol=0, atol=1e-15)
        flops, ntrig = bench.tile_flops(w, computed, skipped)
        assert ntrig == int(trig.sum())
        full = 4 * BM * BN * w.D
        t1 = w.N * sum(-(-((b + 1) * BM) // BN) for b in range(S // BM))
        assert bench.local_tiles(w) == t1
        want = (t1 * w.Z * w.H + int(computed.sum())) * full + int(trig.sum()) * (full // 2)
        assert flops == float(want)
    if BM == BN:
        assert bench.local_tiles(w) == orc.pass1_tiles(L, S, BM)


def test_local_tiles_match_a_brute_force_block_count(bench):
    L, S, BM, BN = 512, 256, 128, 64
    i, j = np.arange(L)[:, None], np.arange(L)[None, :]
    mask = j <= i
    own = 0
    for b in range(L // BM):
        for t in range(L // BN):
            if (t * BN) // S == (b * BM) // S and mask[b * BM:(b + 1) * BM, t * BN:(t + 1) * BN].any():
                own += 1
    assert bench.local_tiles(_w(L, S, BM, BN)) == own


def test_counter_traffic_is_quoted_only_for_the_sources_it_was_measured_on(bench, tmp_path, monkeypatch):
    """A TRAFFIC line of profiles/ is returned while its src= equals the hash of the kernel
    sources in the tree; on any other sources the figure is withheld and marked stale."""
    here = bench.kernel_source_id()
    assert len(here) == 12 and here == bench.kernel_source_id()
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "a.txt").write_text(
        "notes\n"
        f"TRAFFIC workload=w1 tau=0.005 block_m=64 kernel=k1 bytes=123 commit=abc src={here}\n"
        "TRAFFIC workload=w1 tau=0.005 block_m=64 kernel=k2 bytes=456 commit=abc src=000000000000\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_source_id", lambda: here)
    b, src = bench.recorded_traffic("w1", 5e-3, 64, "k1")
    assert b == 123.0 and src["stale"] is False and src["commit"] == "abc" and src["file"].endswith("a.txt")
    b, src = bench.recorded_traffic("w1", 5e-3, 64, "k2")
    assert b is None and src["stale"] is True
    assert bench.recorded_traffic("w1", 5e-3, 128, "k1") == (None, None)
    assert bench.recorded_traffic("w1", 1e-3, 64, "k1") == (None, None)


def test_tracked_traffic_lines_match_the_sources_in_the_tree(bench):
    """The figures bench.py would quote today: every TRAFFIC line on file names the current
    kernel sources (a kernel change without a fresh counter run shows up here, not in a stale
    roofline.traffic)."""
    import glob
    here = bench.kernel_source_id()
    lines = [l for f in glob.glob(os.path.join(ROOT, "profiles", "*.txt")) for l in open(f) if l.startswith("TRAFFIC ")]
    assert lines
    stale = [l for l in lines if f"src={here}" not in l]
    if stale:
        pytest.skip(f"{len(stale)} TRAFFIC line(s) were measured on other kernel sources; bench.py reports them as stale")
