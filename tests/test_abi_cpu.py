"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/comet.h declares, and its host-only entry points (the adaptive error
bound of Sec. 3.2/3.3 and the worst-case size) agree with the oracle.  No device
work is launched here."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def comet():
    from paper_2111_09562_amd import build, comet as libcomet
    build.build()
    libcomet.lib()
    return libcomet


def test_every_declared_symbol_is_exported(comet):
    text = open(os.path.join(ROOT, "include", "comet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(comet_[a-z_0-9]+)\s*\(", text))
    assert declared == set(comet.EXPORTS)
    L = comet.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_adapt_eb_matches_oracle(comet, oracle):
    rng = np.random.default_rng(3)
    assert np.float32(comet.comet_adapt_eb(2e-3, 5e-4, 0.25, 64)) == np.float32(0.03125)
    for _ in range(200):
        M, L = float(rng.uniform(1e-6, 1e-1)), float(rng.uniform(1e-7, 1e-2))
        R, N = float(rng.uniform(0.01, 1.0)), int(rng.integers(1, 1024))
        assert np.float32(comet.comet_adapt_eb(M, L, R, N)) == oracle.adapt_eb(M, L, R, N)
    assert np.float32(comet.comet_adapt_eb(1e-3, 1e-4, 0.5, 32, eb_min=0.5, eb_max=1.0)) == oracle.adapt_eb(1e-3, 1e-4, 0.5, 32, eb_min=0.5, eb_max=1.0)
    assert np.float32(comet.comet_adapt_eb(1e-3, 0.0, 0.5, 32, eb_max=0.25)) == np.float32(0.25)
    for bad in [(float("nan"), 1e-4, 0.5, 32), (1e-3, -1.0, 0.5, 32), (1e-3, 1e-4, 1.5, 32), (1e-3, 1e-4, 0.5, 0)]:
        with pytest.raises(comet.CometError) as ei:
            comet.comet_adapt_eb(*bad)
        assert ei.value.code == comet.ERR_INVALID


def test_controller_matches_oracle(comet, oracle):
    """The active factor W through the C ABI against the oracle's, on random histories of bounds that
    sometimes jump (both directions), sometimes hit a factor of exactly two and mostly stay put."""
    rng = np.random.default_rng(11)
    for w0 in (0, 1, 7, 64):
        a, b = comet.Controller(w0), oracle.Controller(w0)
        assert a.w == b.w == (w0 or 1000)
        eb = rng.uniform(1e-4, 1e-1, 5).astype(np.float32)
        for step in range(400):
            assert a.comet_controller_tick() == b.tick()
            if step % 3 == 0:
                kind = rng.integers(0, 4)
                f = {0: rng.uniform(0.9, 1.1, 5), 1: rng.uniform(0.2, 5.0, 5), 2: np.full(5, 2.0), 3: np.full(5, 0.5)}[int(kind)]
                new = (eb * f.astype(np.float32)).astype(np.float32)
                assert a.comet_controller_update(eb, new) == b.update(eb, new)
                eb = new
    c = comet.Controller(8)
    for bad in ([0.0], [float("nan")], [-1.0], [float("inf")]):
        with pytest.raises(comet.CometError) as ei:
            c.comet_controller_update(bad, [1.0])
        assert ei.value.code == comet.ERR_INVALID


def test_compress_bound_matches_oracle(comet, oracle):
    for shape, nb, cs in [((8, 64, 56, 56), 1024, 128), ((1, 1, 1, 1), 4, 64), ((64, 2048, 7, 7), 65536, 256)]:
        assert comet.comet_compress_bound(shape, nb, cs) == oracle.compress_bound(shape, nb, cs)
    assert comet.comet_compress_bound((0, 1, 1, 1), 1024, 128) == 0
    assert comet.comet_compress_bound((1, 1, 1, 1), 1023, 128) == 0


def test_strerror(comet):
    assert comet.strerror(0) == "ok"
    assert "invalid" in comet.strerror(comet.ERR_INVALID)
