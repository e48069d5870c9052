"""GPU parity: every stage of libcomet and the whole compress / decompress path,
called through the C ABI, compared element by element (bit-exact) with the CPU
oracle on the same seeded inputs.  Tolerance: 0 -- integers, bytes and the fp32
bit patterns of the decompressed values must all be identical (every float step
is a single IEEE operation on both sides, built without contraction).
"""
import numpy as np
import pytest

from paper_2111_09562_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def comet():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2111_09562_amd import comet as libcomet
    libcomet.lib()
    return libcomet


@pytest.fixture(scope="module")
def ctx(comet):
    c = comet.Context(max_elems=8 * 64 * 56 * 56 + 4096, max_nbins=65536)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def oracle_records(oracle, x, eb, nbins):
    q, vflag, nnz = oracle.prequant(x, eb)
    codes, delta = oracle.predict_code(q, x.shape, nbins)
    esc = np.flatnonzero(codes == 0)
    ver = np.flatnonzero(vflag)
    keys = np.concatenate([2 * esc, 2 * ver + 1]).astype(np.uint32)
    vals = np.concatenate([delta[esc].view(np.uint32), x.ravel()[ver].view(np.uint32)])
    order = np.argsort(keys, kind="stable")
    rec = np.stack([keys[order], vals[order]], axis=1).astype(np.uint32)
    return codes, rec, nnz, int(ver.size)


SHAPES = [
    ((2, 8, 56, 56), "blur"), ((3, 5, 17, 13), "blur"), ((1, 1, 1, 1), "blur"), ((4, 33, 7, 7), "blur"),
    ((1, 2, 224, 224), "blur"), ((2, 3, 5, 1), "blur"), ((1, 1, 1, 4099), "blur"), ((2, 2, 112, 112), "lap"),
    ((5, 7, 14, 14), "blur"), ((1, 3, 200, 3), "lap"),
    # planes wider than 512 columns (flat-tile quantise kernel, fused decode + LDS-tile reconstruction): the row
    # above and the up-left neighbour, rows that wrap inside a 16-byte load, the carry between strips of a plane
    ((1, 2, 9, 600), "blur"), ((2, 1, 40, 1030), "blur"), ((1, 1, 3, 8192), "lap"),
]


def make_input(shape, kind, seed):
    if kind == "lap":
        return synth.relu_laplace(shape, seed)
    return synth.relu_blur(shape, seed, blur=3, shift=-0.2)


@pytest.mark.parametrize("shape,kind", SHAPES)
@pytest.mark.parametrize("eb,nbins", [(1e-2, 1024), (1e-3, 1024), (1e-4, 65536), (5e-2, 4)])
def test_stage_quantize(comet, ctx, oracle, shape, kind, eb, nbins):
    x = make_input(shape, kind, seed=31)
    n = x.size
    want_codes, want_rec, want_nnz, want_nv = oracle_records(oracle, x, eb, nbins)
    want_hist = oracle.histogram(want_codes, nbins)
    codes = torch.empty(n + 8, dtype=torch.int16, device="cuda")
    hist = torch.empty(nbins, dtype=torch.int32, device="cuda")
    rec = torch.zeros(2 * (2 * n + 1), dtype=torch.int32, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    ctx.comet_stage_quantize(dev(x), eb, nbins, codes, hist, rec, counts)
    ctx.comet_sync()
    got_counts = counts.cpu().numpy()
    assert got_counts.tolist() == [want_rec.shape[0], want_nv, want_nnz]
    assert np.array_equal(codes.cpu().numpy().view(np.uint16)[:n], want_codes)
    assert np.array_equal(hist.cpu().numpy().view(np.uint32), want_hist)
    got_rec = rec.cpu().numpy().view(np.uint32)[: 2 * want_rec.shape[0]].reshape(-1, 2)
    assert np.array_equal(got_rec, want_rec)


def _hist_cases():
    rng = np.random.default_rng(41)
    cases = {}
    h = np.zeros(1024, np.uint32); act = rng.choice(1024, 300, replace=False); h[act] = rng.geometric(0.001, 300)
    cases["geometric300"] = h
    cases["uniform8"] = np.full(8, 5, np.uint32)
    h = np.zeros(1024, np.uint32); h[rng.choice(1024, 777, replace=False)] = 1 + rng.integers(0, 4, 777)
    cases["many_ties"] = h
    h = np.zeros(16, np.uint32); h[9] = 77
    cases["single"] = h
    fib = [1, 1]
    while len(fib) < 47:
        fib.append(fib[-1] + fib[-2])
    cases["fibonacci47"] = np.array(fib + [0], np.uint32)
    h = np.zeros(4096, np.uint32); h[rng.choice(4096, 3000, replace=False)] = rng.integers(1, 2 ** 20, 3000)
    cases["bins4096"] = h
    h = np.zeros(65536, np.uint32); h[rng.choice(65536, 20000, replace=False)] = rng.geometric(1e-4, 20000)
    cases["bins65536"] = h
    cases["two"] = np.array([0, 3, 0, 9], np.uint32)
    cases["ones1024"] = np.ones(1024, np.uint32)
    return cases


@pytest.mark.parametrize("name", list(_hist_cases().keys()))
def test_stage_codebook(comet, ctx, oracle, name):
    h = _hist_cases()[name]
    nb = h.size
    want_len = oracle.code_lengths(h)
    want_code = oracle.canonical_codes(want_len)
    lens = torch.empty(nb, dtype=torch.uint8, device="cuda")
    codes = torch.empty(nb, dtype=torch.int64, device="cuda")
    ctx.comet_stage_codebook(dev(h.view(np.int32)), nb, lens, codes)
    ctx.comet_sync()
    assert np.array_equal(lens.cpu().numpy(), want_len)
    assert np.array_equal(codes.cpu().numpy().view(np.uint64), want_code)


def test_stage_codebook_sweep(comet, ctx, oracle):
    """Code lengths and canonical codes over many alphabets: every size around the limits of the
    merge rounds (one wavefront in registers, the workgroup, global scratch) and of the counting
    order (by-symbol table up to 8192 bins), weight distributions with few and with many ties,
    counts up to 2^32 - 1."""
    rng = np.random.default_rng(2024)
    cases = []
    for nb in (16, 1024, 2048, 4096, 8192, 16384):
        for m in (2, 3, 31, 63, 64, 65, 127, 129, 700, 1024, 2047, 2048, 2049, 3000):
            if m > nb:
                continue
            for kind in ("zipf", "flat", "expo", "huge"):
                if rng.random() < 0.45 and m not in (64, 65, 2048, 2049):
                    continue
                h = np.zeros(nb, np.uint64)
                act = rng.choice(nb, m, replace=False)
                if kind == "zipf":
                    w = np.floor(1e6 / (1 + rng.permutation(m)) ** 1.3) + 1
                elif kind == "flat":
                    w = rng.integers(1, 4, m)
                elif kind == "expo":
                    w = np.floor(np.exp(rng.uniform(0, 20, m))) + 1
                else:
                    w = rng.integers(2 ** 31, 2 ** 32 - 1, m)
                h[act] = w
                cases.append((nb, m, kind, h.astype(np.uint32)))
    assert len(cases) > 60
    for nb, m, kind, h in cases:
        want_len = oracle.code_lengths(h)
        want_code = oracle.canonical_codes(want_len)
        lens = torch.empty(nb, dtype=torch.uint8, device="cuda")
        codes = torch.empty(nb, dtype=torch.int64, device="cuda")
        ctx.comet_stage_codebook(dev(h.view(np.int32)), nb, lens, codes)
        ctx.comet_sync()
        assert np.array_equal(lens.cpu().numpy(), want_len), (nb, m, kind)
        assert np.array_equal(codes.cpu().numpy().view(np.uint64), want_code), (nb, m, kind)


def test_stage_codebook_large_alphabets(comet, ctx, oracle):
    """Alphabets with more occurring symbols than fit LDS: the leaves are sorted by the tile and merge kernels
    (alphabet sizes that are and are not a whole number of tiles, or a power of two of them), the first merge
    rounds run in global memory and the rest in LDS, the canonical order is counted by symbol."""
    rng = np.random.default_rng(77)
    cases = []
    for nb, m in ((2050, 2049), (3000, 2900), (4096, 4096), (5002, 2500), (8192, 2100), (16384, 9000), (40000, 33000),
                  (65536, 2049), (65536, 26000), (65536, 65536), (65534, 65534)):
        for kind in ("tail", "flat", "expo", "ones"):
            h = np.zeros(nb, np.uint64)
            act = rng.choice(nb, m, replace=False)
            if kind == "tail":                 # what a fine error bound gives: a heavy centre, thousands of symbols seen a few times
                w = np.floor(5e7 * np.exp(-np.abs(act - nb / 2.0) / (nb / 40.0))) + rng.integers(1, 4, m)
            elif kind == "flat":
                w = rng.integers(1, 3, m)
            elif kind == "expo":
                w = np.floor(np.exp(rng.uniform(0, 21, m))) + 1
            else:
                w = np.ones(m)
            h[act] = w
            cases.append((nb, m, kind, h.astype(np.uint32)))
    for nb, m, kind, h in cases:
        want_len = oracle.code_lengths(h)
        want_code = oracle.canonical_codes(want_len)
        lens = torch.empty(nb, dtype=torch.uint8, device="cuda")
        codes = torch.empty(nb, dtype=torch.int64, device="cuda")
        ctx.comet_stage_codebook(dev(h.view(np.int32)), nb, lens, codes)
        ctx.comet_sync()
        assert np.array_equal(lens.cpu().numpy(), want_len), (nb, m, kind)
        assert np.array_equal(codes.cpu().numpy().view(np.uint64), want_code), (nb, m, kind)


def _deep_histogram(levels, nbins):
    """Counts whose Huffman tree is a chain `levels` deep at its far end: Fibonacci numbers as long as they
    fit 32 bits, then groups of equal counts that add up to the next Fibonacci number (a group merges into
    one node before the chain reaches it)."""
    fib = [1, 1]
    while len(fib) < levels + 2:
        fib.append(fib[-1] + fib[-2])
    h = list(fib[:47])
    for j in range(47, levels + 1):
        k = 1
        while fib[j] / k >= 2 ** 32 - 1:
            k *= 2
        h += [fib[j] // k + 1] * k
    assert len(h) <= nbins
    return np.array(h + [0] * (nbins - len(h)), np.uint32)


def test_stage_codebook_longest_code(comet, ctx, oracle):
    """The longest code word either side accepts has 57 bits.  No tensor below 2^31 elements gets there (a leaf
    at depth d needs a total count of Fibonacci(d + 2)); a hand-made histogram does: 57 bits is built and
    equal on both sides, anything deeper is refused by both."""
    h = _deep_histogram(62, 8192)
    want_len = oracle.code_lengths(h)
    assert want_len.max() == 57
    lens = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    codes = torch.empty(h.size, dtype=torch.int64, device="cuda")
    ctx.comet_stage_codebook(dev(h.view(np.int32)), h.size, lens, codes)
    ctx.comet_sync()
    assert np.array_equal(lens.cpu().numpy(), want_len)
    assert np.array_equal(codes.cpu().numpy().view(np.uint64), oracle.canonical_codes(want_len))
    h = _deep_histogram(64, 16384)
    with pytest.raises(oracle.OracleError):
        oracle.code_lengths(h)
    lens = torch.empty(h.size, dtype=torch.uint8, device="cuda")
    ctx.comet_stage_codebook(dev(h.view(np.int32)), h.size, lens)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_sync()
    assert ei.value.code == comet.ERR_INTERNAL


@pytest.mark.parametrize("chunk_syms", [64, 128, 256])
@pytest.mark.parametrize("n,nbins,conc", [(100_003, 1024, 0.05), (1, 16, 1.0), (64 * 256 * 3 + 5, 64, 0.5), (33_000, 65536, 0.001)])
def test_stage_encode_decode(comet, ctx, oracle, chunk_syms, n, nbins, conc):
    rng = np.random.default_rng(n + chunk_syms)
    p = rng.dirichlet(np.full(min(nbins, 4096), conc))
    syms = rng.choice(min(nbins, 4096), size=n, p=p)
    if nbins > 4096:
        syms = syms * (nbins // 4096)        # spread over the alphabet, outside the cached table window
    codes = syms.astype(np.uint16)
    hist = oracle.histogram(codes, nbins)
    ln = oracle.code_lengths(hist)
    cw = oracle.canonical_codes(ln)
    want_off, want_payload = oracle.encode(codes, nbins, chunk_syms, ln, cw)
    # the encode table lives in the context: build it with the codebook stage
    lens_d = torch.empty(nbins, dtype=torch.uint8, device="cuda")
    ctx.comet_stage_codebook(dev(hist.view(np.int32)), nbins, lens_d)
    n_chunks = (n + chunk_syms - 1) // chunk_syms
    off_d = torch.empty(n_chunks, dtype=torch.int32, device="cuda")
    payload_d = torch.zeros(want_payload.size + 16, dtype=torch.int32, device="cuda")
    pw_d = torch.zeros(1, dtype=torch.int64, device="cuda")
    codes_d = torch.zeros(n + 16, dtype=torch.int16, device="cuda")
    codes_d[:n] = dev(codes.view(np.int16))
    ctx.comet_stage_encode(codes_d, n, nbins, chunk_syms, off_d, payload_d, pw_d)
    ctx.comet_sync()
    assert int(pw_d.item()) == want_payload.size
    assert np.array_equal(off_d.cpu().numpy().view(np.uint32), want_off)
    assert np.array_equal(payload_d.cpu().numpy().view(np.uint32)[: want_payload.size], want_payload)
    assert np.array_equal(lens_d.cpu().numpy(), ln)
    # decode the oracle's stream
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    ctx.comet_stage_decode(dev(ln), nbins, dev(want_off.view(np.int32)), dev(want_payload.view(np.int32)),
                           want_payload.size, n, chunk_syms, out)
    ctx.comet_sync()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), codes)


def test_stage_decode_large_alphabet(comet, ctx, oracle):
    """Tens of thousands of active symbols: the canonical order of the decode tables is built over
    several blocks of symbols and kept in global memory, and most codes are longer than the
    look-up table."""
    rng = np.random.default_rng(77)
    nbins, n, chunk_syms = 65536, 300_000, 128
    active = rng.choice(nbins, 20_000, replace=False)
    codes = active[rng.integers(0, active.size, n)].astype(np.uint16)
    codes[:5000] = active[0]                                   # one frequent symbol: code lengths spread out
    hist = oracle.histogram(codes, nbins)
    ln = oracle.code_lengths(hist)
    cw = oracle.canonical_codes(ln)
    want_off, want_payload = oracle.encode(codes, nbins, chunk_syms, ln, cw)
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    ctx.comet_stage_decode(dev(ln), nbins, dev(want_off.view(np.int32)), dev(want_payload.view(np.int32)),
                           want_payload.size, n, chunk_syms, out)
    ctx.comet_sync()
    assert np.array_equal(out.cpu().numpy().view(np.uint16), codes)
    # and through the whole path: a tensor whose residuals spread over a 65536-bin alphabet
    x = (rng.normal(0, 40.0, (2, 3, 64, 96))).astype(np.float32)
    want = oracle.compress(x, 1e-3, 65536, 64)
    assert oracle.parse_container(want)["n_active"] > 2048
    out_c, used = gpu_compress(ctx, comet, x, 1e-3, 65536, 64)
    assert used == want.size and np.array_equal(out_c[:used].cpu().numpy(), want)
    y = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out_c, used, x.shape, y)
    ctx.comet_sync()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), oracle.decompress(want).ravel().view(np.uint32))


def test_stage_decode_long_codes(comet, ctx, oracle):
    fib = [1, 1]
    while len(fib) < 47:
        fib.append(fib[-1] + fib[-2])
    ln = oracle.code_lengths(np.array(fib + [0], np.uint32))
    cw = oracle.canonical_codes(ln)
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 47, size=5000).astype(np.uint16)
    for cs in (33, 64, 100):
        off, payload = oracle.encode(codes, 48, cs, ln, cw)
        out = torch.empty(codes.size, dtype=torch.int16, device="cuda")
        ctx.comet_stage_decode(dev(ln), 48, dev(off.view(np.int32)), dev(payload.view(np.int32)), payload.size, codes.size, cs, out)
        ctx.comet_sync()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), codes)


@pytest.mark.parametrize("shape,kind", SHAPES)
@pytest.mark.parametrize("eb,nbins", [(1e-2, 1024), (1e-3, 256)])
def test_stage_reconstruct(comet, ctx, oracle, shape, kind, eb, nbins):
    x = make_input(shape, kind, seed=51)
    if x.size > 8:
        x.ravel()[3] = np.nan
        x.ravel()[x.size // 2] = 1e30
    codes, rec, _, _ = oracle_records(oracle, x, eb, nbins)
    want = oracle.reconstruct(codes, rec, x.shape, nbins, eb)
    out = torch.empty(x.size, dtype=torch.float32, device="cuda")
    rec_d = dev(rec.view(np.int32).ravel()) if rec.size else None
    ctx.comet_stage_reconstruct(dev(codes.view(np.int16)), rec_d, rec.shape[0], x.shape, nbins, eb, out)
    ctx.comet_sync()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want.ravel().view(np.uint32))


def gpu_compress(ctx, comet, x, eb, nbins, chunk_syms=128, capacity=None):
    ctx.comet_set_chunk_syms(chunk_syms)
    cap = capacity if capacity is not None else comet.comet_compress_bound(x.shape, nbins, chunk_syms)
    out = torch.empty(cap, dtype=torch.uint8, device="cuda")
    used = ctx.comet_compress(dev(x), eb, nbins, out)
    return out, used


@pytest.mark.parametrize("shape,kind", SHAPES)
@pytest.mark.parametrize("eb,nbins,chunk_syms", [(1e-2, 1024, 128), (1e-3, 1024, 64), (1e-4, 65536, 256), (5e-2, 4, 128), (1e-2, 4096, 128)])
def test_compress_container_bytes(comet, ctx, oracle, shape, kind, eb, nbins, chunk_syms):
    x = make_input(shape, kind, seed=61)
    want = oracle.compress(x, eb, nbins, chunk_syms)
    out, used = gpu_compress(ctx, comet, x, eb, nbins, chunk_syms)
    assert used == want.size
    got = out[:used].cpu().numpy()
    assert np.array_equal(got, want)
    info = ctx.comet_peek(out, used)
    assert (info.shape.n, info.shape.c, info.shape.h, info.shape.w) == tuple(x.shape)
    assert info.total_bytes == used and info.nnz == np.count_nonzero(x)


@pytest.mark.parametrize("shape,kind", SHAPES)
@pytest.mark.parametrize("hint", [64, 128])
@pytest.mark.parametrize("eb,nbins,chunk_syms", [(1e-2, 1024, 128), (1e-3, 1024, 77), (1e-4, 65536, 256), (5e-2, 4, 1000), (1e-3, 256, 64)])
def test_decompress_oracle_container(comet, ctx, oracle, shape, kind, eb, nbins, chunk_syms, hint):
    """The decompressor accepts any chunk size: feed it the oracle's container.  `hint` is the chunk size the
    context compresses with, which picks the kernels that are launched: with 64 the single fused kernel and,
    behind it, the general one for containers the fused kernel leaves alone; else the two-kernel path."""
    ctx.comet_set_chunk_syms(hint)
    x = make_input(shape, kind, seed=71)
    if x.size > 100:
        x.ravel()[7] = np.inf
        x.ravel()[50] = -0.0
    buf = oracle.compress(x, eb, nbins, chunk_syms)
    want = oracle.decompress(buf)
    pad = (-buf.size) % 16
    cont = dev(np.concatenate([buf, np.zeros(pad, np.uint8)]))
    out = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(cont, buf.size, x.shape, out)
    ctx.comet_sync()
    got = out.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.ravel().view(np.uint32))
    finite = np.isfinite(x.ravel())
    err = np.abs(got.astype(np.float64)[finite] - x.ravel().astype(np.float64)[finite])
    assert err.max() <= np.float64(np.float32(eb))


def test_which_kernels_decompress(comet, oracle):
    """Chunks of 64 symbols and planes of at most 512 columns take the fused kernel alone; any other chunk size
    under the same context falls to the general kernel behind it; a context set to another chunk size takes
    the two-kernel path.  All give the oracle's values."""
    shape = (2, 8, 56, 56)
    x = synth.relu_blur(shape, seed=44, blur=3, shift=-0.2)
    c = comet.Context(max_elems=x.size, max_nbins=1024)
    c.comet_profile_enable(True)
    FUSED, DECODE, SCAN = 8, 5, 4
    for hint, chunk, want_launches in [(64, 64, (1, 0, 0)), (64, 100, (1, 0, 0)), (128, 64, (0, 1, 1)), (128, 128, (0, 1, 1))]:
        buf = oracle.compress(x, 1e-2, 1024, chunk)
        cont = dev(np.concatenate([buf, np.zeros((-buf.size) % 16, np.uint8)]))
        out = torch.zeros(x.size, dtype=torch.float32, device="cuda")
        c.comet_set_chunk_syms(hint)
        c.comet_profile_reset()
        c.comet_decompress(cont, buf.size, shape, out)
        c.comet_sync()
        got = tuple(c.comet_profile_read(k)[0] for k in (FUSED, DECODE, SCAN))
        assert got == want_launches, (hint, chunk, got)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.decompress(buf).ravel().view(np.uint32)), (hint, chunk)
    c.close()


@pytest.mark.parametrize("shape", [
    (3, 7, 200, 100),      # planes of five strips, two columns per lane: column sums handed from strip to strip and across wavefronts
    (2, 5, 333, 97),       # odd width (one column per lane, two 64-lane segments), strips that end inside planes
    (4, 40, 90, 44),       # 32-lane halves: two runs of rows side by side, plane starts inside a run
    (6, 300, 40, 12),      # narrow planes: eight runs of rows side by side, several planes per run
    (2, 2000, 5, 3),       # tiny planes: many planes per run, rows of three lanes
    (8, 4000, 7, 7),       # ... strips whose rows do not divide evenly among the eight runs (a shorter last run), two strips per segment
    (3, 500, 14, 14),      # ... the same with two columns per lane
    (5, 700, 7, 7),        # ... and with a single short strip
    (1, 3, 1500, 128),     # the widest plane that goes this way
    (2, 3, 300, 130),      # just beyond it with two columns per lane: two segments of 64 lanes, still dealt to all wavefronts
    (3, 5, 60, 256),       # the widest plane that goes this way with two columns per lane
    (2, 3, 150, 129),      # one column per lane beyond 128 columns: a segment per wavefront, sums stay in registers
    (1, 2, 200, 258),      # the same with two columns per lane
    (1, 2, 700, 224),      # four segments of 64 lanes... two columns per lane, planes much larger than a strip
])
def test_fused_decompression_strips(comet, oracle, shape):
    """Decompression in one kernel on shapes whose planes, strips and segments do not line up: planes larger and
    smaller than a strip, strips that end inside planes, escapes (a small alphabet at a tight bound: their
    values come from the list in LDS, and beyond its capacity from the container) and verbatim values on
    both sides of strip boundaries.  Against the oracle, bit for bit; fp32 and bfloat16 outputs."""
    x = synth.relu_blur(shape, seed=sum(shape), blur=3, shift=-0.2)
    flat = x.ravel()
    rng = np.random.default_rng(7)
    for i in rng.integers(0, flat.size, 40):
        flat[i] = [np.inf, -np.inf, 3.0e9, -0.0, np.nan][i % 5]
    ctx = comet.Context(max_elems=x.size, max_nbins=1024)
    ctx.comet_set_chunk_syms(64)
    for eb, nbins in [(1e-2, 1024), (2e-3, 16), (1e-3, 64)]:
        buf = oracle.compress(x, eb, nbins, 64)
        want = oracle.decompress(buf).ravel()
        cont = dev(np.concatenate([buf, np.zeros((-buf.size) % 16, np.uint8)]))
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        ctx.comet_decompress(cont, buf.size, shape, y)
        ctx.comet_sync()
        got = y.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (shape, eb, nbins, int(np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))[0]))
        if shape[3] <= 512:
            y16 = torch.empty(x.size, dtype=torch.bfloat16, device="cuda")
            ctx.comet_decompress_16(cont, buf.size, shape, y16)
            ctx.comet_sync()
            assert np.array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), oracle.narrow16(want, oracle.BF16)), (shape, eb, nbins)
    ctx.close()


# Plane widths on both sides of every boundary between the lane mappings of the quantise and the
# scan kernels (one or two columns per lane; several rows per step up to 32 lanes per row; 1, 2, 4, 8
# segments of 64 lanes), odd and even, with heights that leave a ragged last step and last strip.
WIDTHS = [2, 8, 15, 16, 18, 31, 32, 33, 34, 62, 63, 64, 65, 66, 99, 126, 128, 129, 130, 201, 254, 256, 257, 258, 300, 333, 510, 511, 512]


@pytest.mark.parametrize("w", WIDTHS)
def test_widths_compress_and_decompress(comet, ctx, oracle, w):
    """Container bytes and decompressed bits for one width of every lane mapping, with escapes (a
    small alphabet at a tight bound), verbatim values and negative zero among the inputs."""
    h = 11 if w > 64 else 37
    shape = (2, 3, h, w)
    x = synth.relu_blur(shape, seed=500 + w, blur=3, shift=-0.2)
    flat = x.ravel()
    flat[5 % flat.size] = np.inf
    flat[flat.size // 2] = -np.inf
    flat[flat.size - 1] = np.nan
    flat[flat.size // 3] = -0.0
    flat[flat.size // 5] = 3.0e9                              # beyond the prequantisation range: stored verbatim
    for eb, nbins, chunk in [(1e-2, 1024, 64), (2e-3, 16, 128)]:
        want = oracle.compress(x, eb, nbins, chunk)
        out, used = gpu_compress(ctx, comet, x, eb, nbins, chunk)
        assert used == want.size
        assert np.array_equal(out[:used].cpu().numpy(), want), f"container differs, w={w} eb={eb}"
        want_x = oracle.decompress(want).ravel()
        y = torch.empty(x.size, dtype=torch.float32, device="cuda")
        ctx.comet_decompress(out, used, x.shape, y)
        ctx.comet_sync()
        assert np.array_equal(y.cpu().numpy().view(np.uint32), want_x.view(np.uint32)), f"values differ, w={w} eb={eb}"


# --------------------------------------------------------------------------
# 16-bit activations
# --------------------------------------------------------------------------
def _bits16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("w", [1, 7, 14, 28, 33, 56, 64, 66, 112, 130, 224, 257, 300, 512])
@pytest.mark.parametrize("kind", ["float16", "bfloat16"])
def test_16_bit_compress_and_decompress(comet, ctx, oracle, kind, w):
    """comet_compress_16 writes the container of the widened tensor; comet_decompress_16 returns the
    fp32 reconstruction rounded to the 16-bit type.  Bit-exact against the oracle, every lane mapping,
    with infinities, NaN, negative zero, the largest finite values and subnormals among the inputs."""
    tdt = getattr(torch, kind)
    okind = oracle.F16 if kind == "float16" else oracle.BF16
    h = 9 if w > 64 else 35
    shape = (2, 3, h, w)
    x32 = synth.relu_blur(shape, seed=900 + w, blur=3, shift=-0.2)
    xt = torch.from_numpy(x32).to(tdt)
    flat = xt.view(-1)
    n = flat.numel()
    flat[5 % n] = float("inf")
    flat[n // 2] = float("-inf")
    flat[n - 1] = float("nan")
    flat[n // 3] = -0.0
    flat[n // 5] = torch.finfo(tdt).max
    flat[n // 7] = torch.finfo(tdt).tiny / 4                     # a subnormal of the 16-bit type
    bits = _bits16(xt).reshape(shape)
    xd = xt.cuda()
    for eb, nbins, chunk in [(1e-2, 1024, 64), (2e-3, 16, 128), (1e-3, 4096, 256)]:
        want = oracle.compress_16(bits, okind, eb, nbins, chunk)
        ctx.comet_set_chunk_syms(chunk)
        out = torch.zeros(int(want.size * 1.5) // 16 * 16 + 4096, dtype=torch.uint8, device="cuda")
        used = ctx.comet_compress_16(xd, eb, nbins, out)
        assert used == want.size
        assert np.array_equal(out[:used].cpu().numpy(), want), f"container differs, {kind} w={w} eb={eb}"
        # back in the 16-bit type ...
        y = torch.empty(shape, dtype=tdt, device="cuda")
        ctx.comet_decompress_16(out, used, shape, y)
        ctx.comet_sync()
        got, ref = _bits16(y).ravel(), oracle.decompress_16(want, okind).ravel()
        nan = np.isnan(oracle.widen16(ref, okind))
        assert np.array_equal(got[~nan], ref[~nan]), f"values differ, {kind} w={w} eb={eb}"
        assert np.all(np.isnan(oracle.widen16(got[nan], okind)))
        # ... and as fp32 (the container is an ordinary one)
        y32 = torch.empty(shape, dtype=torch.float32, device="cuda")
        ctx.comet_decompress(out, used, shape, y32)
        ctx.comet_sync()
        assert np.array_equal(y32.cpu().numpy().view(np.uint32).ravel(), oracle.decompress(want).view(np.uint32).ravel())
    ctx.comet_set_chunk_syms(128)


def test_decompress_into_an_output_that_is_not_pair_aligned(comet, ctx, oracle):
    """Even widths take two columns per lane only if every pair of outputs is aligned; an output that
    starts one element into an allocation goes the one-column way and gives the same bits."""
    shape = (2, 3, 20, 56)
    x = synth.relu_blur(shape, seed=77, blur=3, shift=-0.2)
    want = oracle.compress(x, 1e-2, 1024, 64)
    ref = oracle.decompress(want).ravel()
    cont = dev(np.concatenate([want, np.zeros((-want.size) % 16, np.uint8)]))
    n = x.size
    y = torch.empty(n + 1, dtype=torch.float32, device="cuda")[1:]
    assert y.data_ptr() % 8 == 4
    ctx.comet_decompress(cont, want.size, shape, y)
    ctx.comet_sync()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    for tdt, okind in ((torch.float16, oracle.F16), (torch.bfloat16, oracle.BF16)):
        y16 = torch.empty(n + 1, dtype=tdt, device="cuda")[1:]
        assert y16.data_ptr() % 4 == 2
        ctx.comet_decompress_16(cont, want.size, shape, y16)
        ctx.comet_sync()
        assert np.array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), oracle.narrow16(ref, okind))


def test_16_bit_errors(comet, ctx):
    x = torch.zeros((1, 1, 2, 513), dtype=torch.float16, device="cuda")
    out = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(comet.CometError) as e:
        ctx.comet_compress_16(x, 1e-2, 1024, out)                # wider than the row-walking kernels take
    assert e.value.code == comet.ERR_INVALID
    with pytest.raises(TypeError):
        ctx.comet_compress_16(x.float(), 1e-2, 1024, out)
    rc = comet.lib().comet_compress_16(ctx._h, x.data_ptr(), 3, comet._shape((1, 1, 2, 8)), 1e-2, 1024, None, out.data_ptr(), out.numel(), None)
    assert rc == comet.ERR_INVALID                                # no such element type


# --------------------------------------------------------------------------
# code book reuse
# --------------------------------------------------------------------------

def _reuse_case(comet, ctx, oracle, x_old, x_new, eb, nbins, chunk):
    """Compress x_new with the length table of x_old's container on both sides and compare."""
    ctx.comet_set_chunk_syms(chunk)
    first, used_first = gpu_compress(ctx, comet, x_old, eb, nbins, chunk)
    table = first[comet.HEADER_BYTES: comet.HEADER_BYTES + nbins]              # on the device, inside the older container
    out = torch.empty(comet.comet_compress_bound(x_new.shape, nbins, chunk), dtype=torch.uint8, device="cuda")
    try:
        want = oracle.compress_with_lengths(x_new, eb, nbins, chunk, table.cpu().numpy())
    except oracle.OracleError as e:
        assert e.code == oracle.ERR_INVALID                       # an escape is needed and the table has no code word for it
        with pytest.raises(comet.CometError) as ei:
            ctx.comet_compress_with_codebook(dev(x_new), eb, nbins, table, out)
        assert ei.value.code == comet.ERR_CODEBOOK
        return None
    used = ctx.comet_compress_with_codebook(dev(x_new), eb, nbins, table, out)
    assert used == want.size
    assert np.array_equal(out[:used].cpu().numpy(), want)
    y = torch.empty(x_new.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out, used, x_new.shape, y)
    ctx.comet_sync()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), oracle.decompress(want).ravel().view(np.uint32))
    return used


@pytest.mark.parametrize("w", [7, 14, 28, 56, 63, 112, 200, 224, 333, 512])
@pytest.mark.parametrize("eb,nbins,chunk", [(1e-2, 1024, 64), (2e-3, 64, 128), (1e-3, 4096, 256)])
def test_compress_with_codebook_stale_table(comet, ctx, oracle, w, eb, nbins, chunk):
    h = 9 if w > 64 else 31
    x_old = synth.relu_blur((2, 3, h, w), seed=700 + w, blur=3, shift=-0.2)
    x_new = synth.relu_blur((2, 3, h, w), seed=800 + w, blur=2, shift=0.0) * np.float32(1.5)
    x_new.ravel()[3] = np.inf                                     # a verbatim value
    x_new.ravel()[11] = -900.0                                    # residuals far outside the alphabet: escapes
    x_old.ravel()[5] = 1000.0                                     # ... and in the older tensor, so that its table has a code word for them
    assert _reuse_case(comet, ctx, oracle, x_old, x_new, eb, nbins, chunk) is not None


@pytest.mark.parametrize("shape", [(4, 8, 7, 7), (2, 4, 28, 28), (2, 3, 56, 56), (1, 3, 40, 112), (1, 2, 30, 224), (1, 1, 12, 500)])
@pytest.mark.parametrize("eb,nbins", [(1e-2, 1024), (2e-2, 64), (1e-2, 4096)])
def test_fused_decompression_escapes_of_every_size(comet, ctx, oracle, shape, eb, nbins):
    """Escaped residuals of every kind in one tensor: those that fit the 16 bits a residual has in LDS next to
    the table's own (kept in place), those below the table's range and those beyond 16 bits (listed), more of
    them than the list holds in some strips, and verbatim values between them."""
    rng = np.random.default_rng(shape[3] + nbins)
    x = synth.relu_blur(shape, seed=900 + shape[3], blur=3, shift=-0.2)
    flat = x.ravel()
    k = max(8, flat.size // 25)
    idx = rng.choice(flat.size, k, replace=False)
    mag = np.exp(rng.uniform(np.log(0.5), np.log(5000.0), k)).astype(np.float32)       # residuals from tens to hundreds of thousands of steps
    flat[idx] = mag * rng.choice(np.array([-1.0, 1.0], np.float32), k)
    flat[rng.choice(flat.size, 5, replace=False)] = [np.inf, -np.inf, np.nan, 3e30, -1e-30]
    dense = slice(flat.size // 2, flat.size // 2 + min(700, flat.size // 4))            # a run where nearly everything escapes
    flat[dense] = rng.normal(0, 60.0, flat[dense].size).astype(np.float32)
    want = oracle.compress(x, eb, nbins, 64)
    rec = oracle.parse_container(want)["records"]
    vals = rec[rec[:, 0] % 2 == 0][:, 1].view(np.int32)
    assert (vals > 32767).any() and (vals < -2048).any() and ((vals > -2048) & (vals < 32768)).any()
    out, used = gpu_compress(ctx, comet, x, eb, nbins, 64)
    assert used == want.size and np.array_equal(out[:used].cpu().numpy(), want)
    ref = oracle.decompress(want).ravel().view(np.uint32)
    y = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out, used, shape, y)
    ctx.comet_sync()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), ref)
    ctx.comet_set_chunk_syms(128)


# --------------------------------------------------------------------------
# zero chunks (container version 2)
# --------------------------------------------------------------------------

def _sparse_input(shape, seed):
    """Mostly zeros in blobs, one plane of nothing but zeros, a verbatim value inside a run of zeros, and
    the end of the tensor zero (a last chunk that is short and holds the centre code only)."""
    x = synth.relu_blur(shape, seed=seed, blur=3, shift=-1.0)
    x[0, 0] = 0.0
    x.ravel()[7] = np.inf
    x.ravel()[-(min(37, x.size // 2)):] = 0.0
    return x


@pytest.mark.parametrize("shape", [(2, 3, 56, 56), (3, 5, 7, 7), (2, 2, 28, 30), (1, 3, 33, 130), (1, 2, 20, 224), (1, 2, 9, 600),
                                   (1, 2, 3, 8192), (1, 1, 1, 37)])
@pytest.mark.parametrize("eb,nbins,chunk", [(1e-2, 1024, 64), (1e-3, 65536, 64), (1e-2, 1024, 128), (2e-2, 64, 256)])
def test_zero_chunks_container_and_values(comet, ctx, oracle, shape, eb, nbins, chunk):
    """Every compressor and decompressor kernel with chunks that take no words: chunks of 64 symbols (the
    one-kernel decompression), of 128 and 256 (decode and scan apart), planes wider than 512 columns (the
    general kernel); container bytes and values against the oracle's version 2."""
    x = _sparse_input(shape, seed=500 + shape[3])
    want = oracle.compress(x, eb, nbins, chunk, flags=oracle.ZERO_CHUNKS)
    c = oracle.parse_container(want)
    words = np.diff(np.append(c["chunk_off"], c["payload_words"]).astype(np.int64))
    assert c["version"] == 2 and ((words == 0).any() or x.size < 1000)
    ref = oracle.decompress(want).ravel().view(np.uint32)
    ctx.comet_set_zero_chunks(True)
    try:
        out, used = gpu_compress(ctx, comet, x, eb, nbins, chunk)
    finally:
        ctx.comet_set_zero_chunks(False)
    assert used == want.size and np.array_equal(out[:used].cpu().numpy(), want)
    y = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out, used, x.shape, y)              # (the context is back to version 1: the container says what it is)
    ctx.comet_sync()
    assert np.array_equal(y.cpu().numpy().view(np.uint32), ref)
    if shape[3] <= 512:
        for okind, tdt in ((oracle.F16, torch.float16), (oracle.BF16, torch.bfloat16)):
            y16 = torch.empty(x.size, dtype=tdt, device="cuda")
            ctx.comet_decompress_16(out, used, x.shape, y16)
            ctx.comet_sync()
            assert np.array_equal(y16.view(torch.int16).cpu().numpy().view(np.uint16), oracle.decompress_16(want, okind).ravel())
    ctx.comet_set_chunk_syms(128)


def test_zero_chunks_nothing_but_zeros(comet, ctx, oracle):
    for shape, chunk in (((2, 3, 14, 14), 64), ((1, 2, 40, 100), 128), ((1, 1, 2, 700), 64)):
        x = np.zeros(shape, np.float32)
        want = oracle.compress(x, 1e-2, 1024, chunk, flags=oracle.ZERO_CHUNKS)
        assert oracle.parse_container(want)["payload_words"] == 0
        ctx.comet_set_zero_chunks(True)
        try:
            out, used = gpu_compress(ctx, comet, x, 1e-2, 1024, chunk)
        finally:
            ctx.comet_set_zero_chunks(False)
        assert used == want.size and np.array_equal(out[:used].cpu().numpy(), want)
        y = torch.full((x.size,), 7.0, dtype=torch.float32, device="cuda")
        ctx.comet_decompress(out, used, shape, y)
        ctx.comet_sync()
        assert np.array_equal(y.cpu().numpy().view(np.uint32), np.zeros(x.size, np.uint32))
    ctx.comet_set_chunk_syms(128)


@pytest.mark.parametrize("chunk", [64, 100, 256])
def test_zero_chunks_stage_encode_decode(comet, ctx, oracle, chunk):
    rng = np.random.default_rng(chunk)
    n, nbins = 20_000, 256
    codes = np.full(n, nbins // 2, np.uint16)
    busy = rng.random(n // 50) < 0.4                          # runs of 50 symbols that are not all centre
    for k in np.flatnonzero(busy):
        codes[50 * k: 50 * k + 50] = rng.integers(120, 137, 50)
    hist = oracle.histogram(codes, nbins)
    ln = oracle.code_lengths(hist)
    cw = oracle.canonical_codes(ln)
    want_off, want_payload = oracle.encode(codes, nbins, chunk, ln, cw, zero_chunks=True)
    assert (np.diff(np.append(want_off, want_payload.size).astype(np.int64)) == 0).any()
    ctx.comet_set_zero_chunks(True)
    try:
        if chunk != 100:                                      # the encoder takes chunks of 64, 128 and 256 symbols
            lens_d = torch.empty(nbins, dtype=torch.uint8, device="cuda")
            ctx.comet_stage_codebook(dev(hist.view(np.int32)), nbins, lens_d)
            n_chunks = (n + chunk - 1) // chunk
            off_d = torch.empty(n_chunks, dtype=torch.int32, device="cuda")
            payload_d = torch.zeros(want_payload.size + 16, dtype=torch.int32, device="cuda")
            pw_d = torch.zeros(1, dtype=torch.int64, device="cuda")
            codes_d = torch.zeros(n + 16, dtype=torch.int16, device="cuda")
            codes_d[:n] = dev(codes.view(np.int16))
            ctx.comet_stage_encode(codes_d, n, nbins, chunk, off_d, payload_d, pw_d)
            ctx.comet_sync()
            assert int(pw_d.item()) == want_payload.size
            assert np.array_equal(off_d.cpu().numpy().view(np.uint32), want_off)
            assert np.array_equal(payload_d.cpu().numpy().view(np.uint32)[: want_payload.size], want_payload)
        out = torch.empty(n, dtype=torch.int16, device="cuda")
        ctx.comet_stage_decode(dev(ln), nbins, dev(want_off.view(np.int32)), dev(want_payload.view(np.int32)),
                               want_payload.size, n, chunk, out)
        ctx.comet_sync()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), codes)
    finally:
        ctx.comet_set_zero_chunks(False)


def test_compress_with_codebook_more_lengths_than_fit_lds(comet, ctx, oracle):
    """A given table with more than 2048 code words (its canonical codes are then counted by symbol in global memory)."""
    x_old = synth.relu_blur((4, 8, 56, 56), seed=93, blur=3, shift=0.0)
    x_new = synth.relu_blur((4, 8, 56, 56), seed=94, blur=3, shift=0.0)
    x_old.ravel()[5] = 1000.0
    x_new.ravel()[11] = -900.0
    a, used = gpu_compress(ctx, comet, x_old, 1e-4, 8192, 64)
    assert int(np.count_nonzero(a[comet.HEADER_BYTES: comet.HEADER_BYTES + 8192].cpu().numpy())) > 2048
    assert _reuse_case(comet, ctx, oracle, x_old, x_new, 1e-4, 8192, 64) is not None


def test_compress_with_codebook_own_table_is_compress(comet, ctx, oracle):
    x = synth.relu_blur((2, 8, 56, 56), seed=91, blur=3, shift=-0.2)
    a, used_a = gpu_compress(ctx, comet, x, 1e-2, 1024, 64)
    table = a[comet.HEADER_BYTES: comet.HEADER_BYTES + 1024]
    b = torch.empty_like(a)
    used_b = ctx.comet_compress_with_codebook(dev(x), 1e-2, 1024, table, b)
    assert used_b == used_a and torch.equal(a[:used_a], b[:used_b])


def test_compress_with_codebook_errors(comet, ctx, oracle):
    x = synth.relu_blur((1, 2, 20, 20), seed=92)
    out = torch.empty(comet.comet_compress_bound(x.shape, 64, 64), dtype=torch.uint8, device="cuda")
    ctx.comet_set_chunk_syms(64)
    # smooth older tensor without any escape, newer one with outliers: no code word for the escape it needs
    smooth = np.full((1, 2, 20, 20), 0.25, np.float32)
    rough = x.copy(); rough.ravel()[7] = 50.0
    assert _reuse_case(comet, ctx, oracle, smooth, rough, 1e-2, 64, 64) is None
    for bad in ([2, 1] + [0] * 62, [1, 1, 1] + [0] * 61, [0] * 64, [1, 58] + [0] * 62):      # incomplete, over-full, empty, too long
        t = dev(np.array(bad, np.uint8))
        with pytest.raises(comet.CometError) as ei:
            ctx.comet_compress_with_codebook(dev(x), 1e-2, 64, t, out)
        assert ei.value.code == comet.ERR_CODEBOOK
        with pytest.raises(oracle.OracleError):
            oracle.compress_with_lengths(x, 1e-2, 64, 64, np.array(bad, np.uint8))
    # the context still works afterwards
    used = ctx.comet_compress(dev(x), 1e-2, 64, out)
    assert np.array_equal(out[:used].cpu().numpy(), oracle.compress(x, 1e-2, 64, 64))
    # limits of the entry point: alphabet and plane width
    big = torch.zeros(16384, dtype=torch.uint8, device="cuda")
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_compress_with_codebook(dev(x), 1e-2, 16384, big, torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == comet.ERR_INVALID
    wide = np.zeros((1, 1, 2, 600), np.float32)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_compress_with_codebook(dev(wide), 1e-2, 64, dev(np.array([1, 1] + [0] * 62, np.uint8)), out)
    assert ei.value.code == comet.ERR_INVALID


def test_compress_with_codebook_zero_chunks(comet, ctx, oracle):
    """Container version 2 from the single-pass compressor: with the tensor's own table it is the oracle's version 2."""
    x = synth.relu_blur((2, 8, 56, 56), seed=95, blur=3, shift=-0.2)
    x[1, 2:6] = 0.0                                              # whole planes of zeros: chunks of nothing but the centre code
    want = oracle.compress(x, 1e-2, 1024, 64, flags=oracle.ZERO_CHUNKS)
    a, used_a = gpu_compress(ctx, comet, x, 1e-2, 1024, 64)
    table = a[comet.HEADER_BYTES: comet.HEADER_BYTES + 1024]
    b = torch.empty_like(a)
    ctx.comet_set_zero_chunks(True)
    try:
        used_b = ctx.comet_compress_with_codebook(dev(x), 1e-2, 1024, table, b)
    finally:
        ctx.comet_set_zero_chunks(False)
    assert used_b == want.size and used_b < used_a
    assert np.array_equal(b[:used_b].cpu().numpy(), want)


def test_compress_with_codebook_table_that_expands_the_data(comet, ctx, oracle):
    """The single-pass compressor gives a run of rows 16 bits per symbol of work space.  A table that needs more
    (here: 20 bits for the centre code of a tensor of zeros) is refused with the error that tells the caller to
    compress in full, as for a missing escape code; the oracle, which has no such limit, encodes it.  With zero
    chunks the same tensor takes no words at all and goes through."""
    nbins = 64
    lens = np.zeros(nbins, np.uint8)
    lens[nbins // 2] = 20; lens[0] = 20                           # centre and escape: 20 bits each
    lens[1:20] = np.arange(1, 20, dtype=np.uint8)                 # 2^-1 + ... + 2^-19 + 2 * 2^-20 = 1
    x = np.zeros((1, 4, 32, 32), np.float32)
    oracle.compress_with_lengths(x, 1e-2, nbins, 64, lens)        # valid for the oracle
    out = torch.empty(comet.comet_compress_bound(x.shape, nbins, 64), dtype=torch.uint8, device="cuda")
    ctx.comet_set_chunk_syms(64)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_compress_with_codebook(dev(x), 1e-2, nbins, dev(lens), out)
    assert ei.value.code == comet.ERR_CODEBOOK
    ctx.comet_set_zero_chunks(True)
    try:
        used = ctx.comet_compress_with_codebook(dev(x), 1e-2, nbins, dev(lens), out)
    finally:
        ctx.comet_set_zero_chunks(False)
    y = torch.full((x.size,), 7.0, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out, used, x.shape, y)
    ctx.comet_sync()
    assert not y.any()
    # the context still works afterwards
    used = ctx.comet_compress(dev(x), 1e-2, nbins, out)
    assert np.array_equal(out[:used].cpu().numpy(), oracle.compress(x, 1e-2, nbins, 64))


def test_compress_with_codebook_capacity(comet, ctx, oracle):
    """A container buffer that is too small for the payload: the kernel that moves the words to their place reports it."""
    x = synth.relu_blur((2, 8, 56, 56), seed=96, blur=3, shift=-0.2)
    a, used = gpu_compress(ctx, comet, x, 1e-2, 1024, 64)
    table = a[comet.HEADER_BYTES: comet.HEADER_BYTES + 1024].clone()
    small = torch.zeros((used - 4096) // 16 * 16 + 64, dtype=torch.uint8, device="cuda")
    guard = small[-64:]                                          # not part of the capacity handed over: must stay untouched
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_compress_with_codebook(dev(x), 1e-2, 1024, table, small[:-64])
    assert ei.value.code == comet.ERR_CAPACITY
    assert not guard.any()
    b = torch.empty_like(a)
    assert ctx.comet_compress_with_codebook(dev(x), 1e-2, 1024, table, b) == used and torch.equal(a[:used], b[:used])


def test_abs_mean(comet, ctx, oracle):
    """The controller's statistic.  Tolerance: both sides add non-negative fp64 terms, the oracle in index
    order, the GPU in a fixed tree; each addition is within 2^-53 relative, so the two sums differ by at
    most about n * 2^-53 relative (1.2e-10 at a million terms); 1e-9 is asked for.  Repeated calls must
    give the same bits."""
    for n, seed in [(1, 1), (63, 2), (16384, 3), (1_000_003, 4)]:
        x = (synth.relu_laplace((1, 1, 1, n), seed) - np.float32(0.05)).ravel()
        got = ctx.comet_abs_mean(dev(x))
        want = oracle.abs_mean(x)
        assert abs(got - want) <= 1e-9 * want
        assert ctx.comet_abs_mean(dev(x)) == got
    assert ctx.comet_abs_mean(dev(np.full(4099, -0.375, np.float32))) == 0.375
    assert ctx.comet_abs_mean(dev(np.array([1.0, -np.inf, 2.0], np.float32))) == np.inf
    with pytest.raises(comet.CometError):
        ctx.comet_abs_mean(torch.empty(0, dtype=torch.float32, device="cuda"))


def test_saved_activation_hook_on_a_toy_conv_stack(comet, oracle):
    """Sec. 3.4 end to end on three random conv + ReLU layers: the forward result is untouched, every
    activation saved for backward goes through libcomet (and comes back as the oracle says it must),
    the weight gradients move with the error bound and the containers are smaller than the tensors."""
    from paper_2111_09562_amd.autograd import saved_activations
    torch.manual_seed(0)
    net = torch.nn.Sequential(
        torch.nn.Conv2d(8, 16, 3, padding=1), torch.nn.ReLU(),
        torch.nn.Conv2d(16, 16, 3, padding=1), torch.nn.ReLU(),
        torch.nn.Conv2d(16, 4, 3, padding=1)).cuda()
    x = torch.randn(8, 8, 48, 48, device="cuda")

    def run(hook):
        net.zero_grad(set_to_none=True)
        if hook is None:
            loss = net(x).square().mean()
        else:
            with hook:
                loss = net(x).square().mean()
        loss.backward()
        return float(loss.detach()), [p.grad.detach().clone() for p in net.parameters()]

    base_loss, base = run(None)
    c = comet.Context(max_elems=8 * 16 * 48 * 48, max_nbins=1024)
    c.comet_set_chunk_syms(64)
    errs = []
    for eb in (5e-2, 5e-3):
        hook = saved_activations(c, eb, nbins=1024, min_elems=1 << 12)
        loss, grads = run(hook)
        c.comet_sync()
        assert loss == base_loss                                         # the forward pass does not see the codec
        assert hook.packed >= 3 and hook.unpacked >= hook.packed         # the input and the two ReLU outputs at least
        assert hook.bytes_kept < hook.bytes_in
        errs.append(max(float((g - b).abs().max() / b.abs().max()) for g, b in zip(grads, base)))
    assert errs[0] < 0.2 and errs[1] < 0.5 * errs[0]
    # white noise at a tight bound does not fit 60 % of its size: the hook keeps such a tensor as it is
    hook = saved_activations(c, 1e-5, min_elems=1 << 12)
    assert hook._pack(x) is x and hook.kept_raw == 1
    c.comet_sync()
    # what comes back for one saved tensor is what the oracle decompresses from the oracle's container
    hook = saved_activations(c, 1e-2, min_elems=1 << 12)
    packed = hook._pack(x)
    back = hook._unpack(packed)
    c.comet_sync()
    want = oracle.decompress(oracle.compress(x.cpu().numpy(), 1e-2, 1024, 64))
    assert np.array_equal(back.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # a 16-bit activation comes back in its own type, as the oracle rounds it
    for tdt, okind in ((torch.float16, oracle.F16), (torch.bfloat16, oracle.BF16)):
        x16 = x.to(tdt)
        back = hook._unpack(hook._pack(x16))
        c.comet_sync()
        assert back.dtype == tdt
        bits = x16.view(torch.int16).cpu().numpy().view(np.uint16)
        want = oracle.decompress_16(oracle.compress_16(bits, okind, 1e-2, 1024, 64), okind)
        assert np.array_equal(back.view(torch.int16).cpu().numpy().view(np.uint16), want)
    c.close()


def test_saved_activation_hook_asynchronous(comet, oracle):
    """exact_size=False never waits for a compression.  A container that fits stands in for the tensor and
    decompresses to what the oracle says; one that outgrows its buffer (white noise at a tight bound, the
    low-ratio case of Sec. 3.4) is noticed from its header and the tensor comes back untouched -- never
    an uninitialised buffer -- and the context is left without a latched error."""
    from paper_2111_09562_amd.autograd import saved_activations
    shape = (4, 8, 48, 48)
    c = comet.Context(max_elems=int(np.prod(shape)), max_nbins=1024)
    c.comet_set_chunk_syms(64)
    smooth = torch.from_numpy(synth.relu_blur(shape, seed=5, blur=3, shift=-0.2)).cuda()
    noise = torch.randn(shape, device="cuda", generator=torch.Generator("cuda").manual_seed(1))
    hook = saved_activations(c, 1e-2, min_elems=1 << 12, exact_size=False)
    p1 = hook._pack(smooth)
    back = hook._unpack(p1)
    c.comet_sync()
    want = oracle.decompress(oracle.compress(smooth.cpu().numpy(), 1e-2, 1024, 64))
    assert np.array_equal(back.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert p1.raw is None and hook.packed == 1 and hook.kept_raw == 0
    hook = saved_activations(c, 1e-5, min_elems=1 << 12, exact_size=False)
    p2 = hook._pack(noise)
    back = hook._unpack(p2)
    assert back.data_ptr() == noise.data_ptr() and torch.equal(back, noise)
    assert hook.kept_raw == 1 and hook.packed == 0 and hook.unpacked == 0
    c.comet_sync()                                                  # nothing left latched
    # and inside autograd: gradients through the asynchronous hook equal those through the waiting one
    # (up to the summation order of the convolution's own backward kernels)
    torch.manual_seed(1)
    conv = torch.nn.Conv2d(8, 8, 3, padding=1).cuda()
    grads = []
    for exact in (True, False):
        conv.zero_grad(set_to_none=True)
        with saved_activations(c, 1e-2, min_elems=1 << 12, exact_size=exact):
            loss = conv(torch.relu(conv(smooth))).square().mean()
        loss.backward()
        grads.append(conv.weight.grad.detach().clone())
    c.comet_sync()
    assert torch.allclose(grads[0], grads[1], rtol=1e-4, atol=1e-7)
    c.close()


def test_calls_can_be_captured_in_a_graph(comet, oracle):
    """The asynchronous calls issue kernels only (no memset, no synchronisation), so a stream capture
    records them.  The graph is replayed several times on new inputs, with eager work between the
    replays, and every replay is compared with the oracle."""
    shape = (4, 16, 56, 56)
    c = comet.Context(int(np.prod(shape)), 1024)
    c.comet_set_chunk_syms(64)
    x = torch.empty(shape, dtype=torch.float32, device="cuda")
    cont = torch.zeros(int(x.numel() * 4 * 0.8) // 16 * 16, dtype=torch.uint8, device="cuda")
    y = torch.empty_like(x)
    inputs = [synth.relu_blur(shape, seed=s, blur=3, shift=-0.2) for s in (1, 2, 3)]
    x.copy_(torch.from_numpy(inputs[0]))
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        c.comet_compress(x, 1e-2, 1024, cont, stream=st, sync=False)           # warm-up outside the capture
        c.comet_decompress(cont, cont.numel(), shape, y, stream=st)
        c.comet_sync(st)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            c.comet_compress(x, 1e-2, 1024, cont, stream=torch.cuda.current_stream(), sync=False)
            c.comet_decompress(cont, cont.numel(), shape, y, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for xn in inputs + inputs[:1]:
        x.copy_(torch.from_numpy(xn))
        cont.zero_()
        y.zero_()
        float((x * 2).sum())                                                   # eager work between the replays
        g.replay()
        torch.cuda.synchronize()
        want = oracle.compress(xn, 1e-2, 1024, 64)
        used = int(c.comet_peek(cont, cont.numel()).total_bytes)
        assert used == want.size and np.array_equal(cont[:used].cpu().numpy(), want)
        assert np.array_equal(y.cpu().numpy().view(np.uint32), oracle.decompress(want).view(np.uint32))
    c.comet_sync()
    c.close()


def test_roundtrip_config0_and_determinism(comet, ctx, oracle):
    e = synth.config0()[0]
    x = synth.make(e)
    want = oracle.compress(x, e["eb"], e["nbins"], 128)
    outs = []
    for _ in range(3):
        out, used = gpu_compress(ctx, comet, x, e["eb"], e["nbins"], 128)
        outs.append(out[:used].cpu().numpy())
    assert all(np.array_equal(o, want) for o in outs)
    cont = torch.zeros((want.size + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
    cont[: want.size] = dev(outs[0])
    xh = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(cont, want.size, x.shape, xh)
    ctx.comet_sync()
    got = xh.cpu().numpy().reshape(x.shape)
    assert np.array_equal(got.view(np.uint32), oracle.decompress(want).view(np.uint32))
    assert np.abs(got.astype(np.float64) - x.astype(np.float64)).max() <= np.float64(np.float32(e["eb"]))
    assert np.all(got[x == 0] == 0)


def test_special_values_roundtrip(comet, ctx, oracle):
    x = synth.relu_blur((2, 3, 28, 28), seed=81)
    f = x.ravel()
    f[0] = np.nan; f[1] = np.inf; f[2] = -np.inf; f[3] = 1e30; f[4] = -0.0; f[100] = -3.25; f[-1] = np.nan
    want = oracle.compress(x, 1e-2, 1024, 128)
    out, used = gpu_compress(ctx, comet, x, 1e-2, 1024, 128)
    assert np.array_equal(out[:used].cpu().numpy(), want)
    xh = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(out, used, x.shape, xh)
    ctx.comet_sync()
    assert np.array_equal(xh.cpu().numpy().view(np.uint32), oracle.decompress(want).ravel().view(np.uint32))


def test_all_outliers_worst_case(comet, ctx, oracle):
    x = np.full((1, 2, 16, 16), np.nan, np.float32)
    rng = np.random.default_rng(5)
    x[0, 1] = rng.standard_normal((16, 16)).astype(np.float32) * 1e6
    want = oracle.compress(x, 1e-4, 4, 64)
    out, used = gpu_compress(ctx, comet, x, 1e-4, 4, 64)
    assert used == want.size and used <= comet.comet_compress_bound(x.shape, 4, 64)
    assert np.array_equal(out[:used].cpu().numpy(), want)


def test_capacity_error_and_recovery(comet, ctx, oracle):
    x = synth.relu_blur((2, 4, 56, 56), seed=91)
    want = oracle.compress(x, 1e-3, 1024, 128)
    for cap in (want.size - 16, want.size // 2, 4096, 256):
        with pytest.raises(comet.CometError) as ei:
            gpu_compress(ctx, comet, x, 1e-3, 1024, 128, capacity=cap // 16 * 16)
        assert ei.value.code == comet.ERR_CAPACITY
    # the context keeps working, and an exact-size buffer is enough
    out, used = gpu_compress(ctx, comet, x, 1e-3, 1024, 128, capacity=(want.size + 15) // 16 * 16)
    assert np.array_equal(out[:used].cpu().numpy(), want)


def test_asynchronous_capacity_error_is_latched(comet, ctx, oracle):
    """bytes_out == NULL: nothing is reported by the call itself; the pack kernel seals the header with a
    non-zero status and latches the error, comet_sync returns it once, a decompression of that buffer is
    refused, and the next synchronising compression is clean again."""
    x = synth.relu_blur((2, 4, 56, 56), seed=93)
    want = oracle.compress(x, 1e-3, 1024, 64)
    ctx.comet_set_chunk_syms(64)
    xd = dev(x)
    small = torch.zeros(want.size // 2 // 16 * 16, dtype=torch.uint8, device="cuda")
    guard = small.numel() - 64
    assert ctx.comet_compress(xd, 1e-3, 1024, small[:guard], sync=False) is None
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_sync()
    assert ei.value.code == comet.ERR_CAPACITY
    ctx.comet_sync()                                            # reported once
    assert int(small[guard:].max()) == 0                        # nothing written past the capacity given
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_peek(small, guard)                            # the header says the container is not complete
    assert ei.value.code == comet.ERR_FORMAT
    xh = torch.empty(x.size, dtype=torch.float32, device="cuda")
    ctx.comet_decompress(small, guard, x.shape, xh)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_sync()
    assert ei.value.code == comet.ERR_FORMAT
    # an error latched by an asynchronous call is also returned by the next synchronising compression,
    # which still delivers its own size
    ctx.comet_compress(xd, 1e-3, 1024, small[:guard], sync=False)
    big = torch.zeros((want.size + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
    used = comet.C.c_uint64()
    rc = comet.lib().comet_compress(ctx._h, comet._ptr(xd), comet._shape(x.shape), comet.C.c_float(1e-3), 1024,
                                    comet._stream(None), comet._ptr(big), big.numel(), comet.C.byref(used))
    assert rc == comet.ERR_CAPACITY and used.value == want.size
    assert np.array_equal(big[:want.size].cpu().numpy(), want)
    ctx.comet_sync()


def test_decompress_refuses_a_tensor_larger_than_the_context(comet, oracle):
    """The work buffer of a context holds max_elems residuals: a larger shape is an error before any launch."""
    small = comet.Context(max_elems=1000, max_nbins=1024)
    x = synth.relu_blur((1, 2, 30, 30), seed=94)
    buf = oracle.compress(x, 1e-2, 1024, 64)
    cont = dev(np.concatenate([buf, np.zeros((-buf.size) % 16, np.uint8)]))
    out = torch.empty(x.size, dtype=torch.float32, device="cuda")
    with pytest.raises(comet.CometError) as ei:
        small.comet_decompress(cont, buf.size, x.shape, out)
    assert ei.value.code == comet.ERR_NOMEM
    with pytest.raises(comet.CometError) as ei:
        small.comet_compress(dev(x), 1e-2, 1024, torch.empty(1 << 16, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == comet.ERR_NOMEM
    small.comet_sync()
    small.close()


def test_header_constants_are_checked(comet, ctx, oracle):
    """A header whose reciprocal 1 / (2 eb) does not belong to its eb is refused, as the oracle refuses it."""
    x = synth.relu_blur((1, 4, 28, 28), seed=95)
    buf = oracle.compress(x, 1e-2, 1024, 64)
    bad = buf.copy()
    bad[48:52] = np.array([np.float32(49.0)], np.float32).view(np.uint8)      # r_bits (1 / 0.02 rounds to 50)
    with pytest.raises(oracle.OracleError):
        oracle.decompress(bad)
    xh = torch.empty(x.size, dtype=torch.float32, device="cuda")
    pad = np.zeros((-buf.size) % 16, np.uint8)
    ctx.comet_decompress(dev(np.concatenate([bad, pad])), buf.size, x.shape, xh)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_sync()
    assert ei.value.code == comet.ERR_FORMAT
    ctx.comet_decompress(dev(np.concatenate([buf, pad])), buf.size, x.shape, xh)
    ctx.comet_sync()
    assert np.array_equal(xh.cpu().numpy().view(np.uint32), oracle.decompress(buf).ravel().view(np.uint32))


def test_format_errors(comet, ctx, oracle):
    x = synth.relu_blur((1, 4, 28, 28), seed=92)
    out, used = gpu_compress(ctx, comet, x, 1e-2, 1024, 128)
    xh = torch.empty(x.size, dtype=torch.float32, device="cuda")
    bad = out.clone()
    bad[0] = 0x58
    ctx.comet_decompress(bad, used, x.shape, xh)
    with pytest.raises(comet.CometError) as ei:
        ctx.comet_sync()
    assert ei.value.code == comet.ERR_FORMAT
    ctx.comet_decompress(out, used, (1, 4, 28, 14), torch.empty(x.size // 2, dtype=torch.float32, device="cuda"))
    with pytest.raises(comet.CometError):
        ctx.comet_sync()
    ctx.comet_decompress(out, used - 4, x.shape, xh)          # truncated
    with pytest.raises(comet.CometError):
        ctx.comet_sync()
    ctx.comet_decompress(out, used, x.shape, xh)              # still fine afterwards
    ctx.comet_sync()
    for eb in (0.0, float("nan"), 1e-40):
        with pytest.raises(comet.CometError) as ei:
            gpu_compress(ctx, comet, x, eb, 1024)
        assert ei.value.code == comet.ERR_INVALID
    for nb in (2, 1023, 65538):
        with pytest.raises(comet.CometError):
            gpu_compress(ctx, comet, x, 1e-2, nb)
