"""GPU parity at the full sizes of the benchmark configurations, through the C ABI.

Configs 1-3 are small enough for the CPU oracle to process whole (seconds per
tensor), so containers and decompressed values are compared bit for bit.
Config 1 runs in the launch configuration `bench.py` times: five contexts on
five streams, every call asynchronous, chunks of 64 symbols.
Config 4 (two tensors of 411 M elements, 65536 bins) goes through the oracle
whole as well (about a minute of CPU per tensor, both at once on two threads):
container bytes and every decompressed bit, each tensor alone and with the two
streams overlapped.  Config 3 runs its primary curve and every secondary cell
(each error bound with 1024 and with 65536 bins).
"""
import sys
import time
from concurrent.futures import ThreadPoolExecutor

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


def _progress(request, text):
    """One line past pytest's capture: the long tests say which step they have finished."""
    capman = request.config.pluginmanager.getplugin("capturemanager")
    with capman.global_and_fixture_disabled():
        print(f"\n[{time.strftime('%H:%M:%S')}] {text}", end="", flush=True)


def _check_layer(oracle, x, entry, chunk, cont, out):
    """Container bytes and decompressed bits against the oracle."""
    want = oracle.compress(x, entry["eb"], entry["nbins"], chunk)
    info_bytes = want.size
    got = cont[:info_bytes].cpu().numpy()
    assert np.array_equal(got, want), f"container differs for {entry['shape']}"
    want_x = oracle.decompress(want).ravel()
    got_x = out.cpu().numpy().ravel()
    assert np.array_equal(got_x.view(np.uint32), want_x.view(np.uint32)), f"values differ for {entry['shape']}"
    finite = np.isfinite(x.ravel())
    err = np.abs(got_x.astype(np.float64)[finite] - x.ravel().astype(np.float64)[finite]).max()
    assert err <= np.float64(np.float32(entry["eb"]))
    return info_bytes


def test_config1_full_size_in_bench_configuration(comet, oracle):
    layers = synth.config1(64)
    xs_host = [synth.make(e) for e in layers]
    xs = [torch.from_numpy(x).cuda() for x in xs_host]
    n_ctx = len(layers)
    ctxs = [comet.Context(max_elems=max(x.numel() for x in xs), max_nbins=1024) for _ in range(n_ctx)]
    for c in ctxs:
        c.comet_set_chunk_syms(64)
    streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(n_ctx - 1)]
    conts = [torch.empty(int(x.numel() * 4 * 0.6) // 16 * 16, dtype=torch.uint8, device="cuda") for x in xs]
    outs = [torch.empty_like(x) for x in xs]
    torch.cuda.synchronize()
    for rep in range(2):                                      # a second step reuses every workspace
        for i, (x, e, c) in enumerate(zip(xs, layers, conts)):
            ctxs[i].comet_compress(x, e["eb"], e["nbins"], c, stream=streams[i], sync=False)
        for i in reversed(range(len(xs))):
            ctxs[i].comet_decompress(conts[i], conts[i].numel(), xs[i].shape, outs[i], stream=streams[i])
    for c, st in zip(ctxs, streams):
        c.comet_sync(st)
    total = 0
    for x, e, c, o, ctx in zip(xs_host, layers, conts, outs, ctxs):
        used = int(ctx.comet_peek(c, c.numel()).total_bytes)
        assert used == _check_layer(oracle, x, e, 64, c, o)
        total += used
    assert 3.5 < sum(x.nbytes for x in xs_host) / total < 5.0   # the set compresses about 4.1x
    for c in ctxs:
        c.close()


def test_config1_full_size_bfloat16(comet, oracle):
    """The benchmark set rounded to bfloat16 through comet_compress_16 / comet_decompress_16, five
    contexts on five streams as `bench.py` runs it: containers and 16-bit outputs bit for bit."""
    layers = synth.config1(64)
    xs16 = [torch.from_numpy(synth.make(e)).to(torch.bfloat16) for e in layers]
    bits = [x.view(torch.int16).numpy().view(np.uint16) for x in xs16]
    xs = [x.cuda() for x in xs16]
    n_ctx = len(layers)
    ctxs = [comet.Context(max_elems=max(x.numel() for x in xs), max_nbins=1024) for _ in range(n_ctx)]
    for c in ctxs:
        c.comet_set_chunk_syms(64)
    streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(n_ctx - 1)]
    conts = [torch.empty(int(x.numel() * 4 * 0.6) // 16 * 16, dtype=torch.uint8, device="cuda") for x in xs]
    outs = [torch.empty_like(x) for x in xs]
    torch.cuda.synchronize()
    for i, (x, e, c) in enumerate(zip(xs, layers, conts)):
        ctxs[i].comet_compress_16(x, e["eb"], e["nbins"], c, stream=streams[i], sync=False)
    for i in reversed(range(n_ctx)):
        ctxs[i].comet_decompress_16(conts[i], conts[i].numel(), xs[i].shape, outs[i], stream=streams[i])
    for c, st in zip(ctxs, streams):
        c.comet_sync(st)
    for b, e, cont, out in zip(bits, layers, conts, outs):
        want = oracle.compress_16(b, oracle.BF16, e["eb"], e["nbins"], 64)
        assert np.array_equal(cont[:want.size].cpu().numpy(), want), f"container differs for {e['shape']}"
        got = out.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, oracle.decompress_16(want, oracle.BF16)), f"values differ for {e['shape']}"
    for c in ctxs:
        c.close()


def test_codebook_reuse_full_size(comet, oracle):
    """Code book reuse at the benchmark's sizes.  With a tensor's own table the container must be the one
    comet_compress writes, byte for byte (that one is checked against the oracle above); with the table of a
    different tensor of the layer the values that come back must be the same and the size close (or the call
    reports that the older table has no code word for the escapes the newer tensor needs).  The last case is
    a tensor twice the size of the largest layer."""
    layers = synth.config1(64)
    cases = [(synth.make(e), e["eb"], e["nbins"]) for e in layers]
    big = dict(layers[0]); big["shape"] = (64, 64, 160, 160)                  # 104.9 M elements
    cases.append((synth.make(big), big["eb"], big["nbins"]))
    ctx = comet.Context(max_elems=max(x.size for x, _, _ in cases), max_nbins=1024)
    ctx.comet_set_chunk_syms(64)
    for x, eb, nbins in cases:
        xd = torch.from_numpy(x).cuda()
        a = torch.empty(int(x.size * 4 * 0.6) // 16 * 16, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        used_a = ctx.comet_compress(xd, eb, nbins, a)
        table = a[comet.HEADER_BYTES: comet.HEADER_BYTES + nbins].clone()
        used_b = ctx.comet_compress_with_codebook(xd, eb, nbins, table, b)
        assert used_b == used_a and torch.equal(a[:used_a], b[:used_b]), f"own table, {x.shape}"
        # another tensor of the same kind (the batch reversed and scaled a little): stale table
        xs = torch.flip(xd, dims=[0]) * 1.1
        ya, yb = torch.empty_like(xs), torch.empty_like(xs)
        used_c = ctx.comet_compress(xs, eb, nbins, a)
        ctx.comet_decompress(a, used_c, xs.shape, ya)
        try:
            used_d = ctx.comet_compress_with_codebook(xs, eb, nbins, table, b)
        except comet.CometError as e:
            # new symbols, and the older tensor had no escape, so its table has no code word for one
            assert e.code == comet.ERR_CODEBOOK and int(table[0]) == 0, f"stale table, {x.shape}"
        else:
            assert int(table[0]) != 0 or used_d > 0
            ctx.comet_decompress(b, used_d, xs.shape, yb)
            ctx.comet_sync()
            assert torch.equal(ya.view(torch.int32), yb.view(torch.int32)), f"stale table, {x.shape}"
            assert used_d >= used_c - 4096 and used_d < 1.1 * used_c
        del xd, xs, ya, yb, a, b
    ctx.close()


def test_config2_full_size(comet, oracle):
    layers = synth.config2(32)
    ctx = comet.Context(max_elems=max(int(np.prod(e["shape"])) for e in layers), max_nbins=4096)
    for e in layers:
        x = synth.make(e)
        xd = torch.from_numpy(x).cuda()
        cont = torch.empty(x.nbytes // 2 // 16 * 16, dtype=torch.uint8, device="cuda")
        out = torch.empty_like(xd)
        used = ctx.comet_compress(xd, e["eb"], e["nbins"], cont)
        ctx.comet_decompress(cont, used, x.shape, out)
        ctx.comet_sync()
        assert used == _check_layer(oracle, x, e, 64, cont, out)
        del xd, cont, out
    ctx.close()


def test_config3_eb_sweep_and_adaptive_bound(comet, oracle, request):
    entries = synth.config3(64)
    x = synth.make(entries[0])
    xd = torch.from_numpy(x).cuda()
    ctx = comet.Context(max_elems=x.size, max_nbins=65536)
    cont = torch.empty(x.nbytes, dtype=torch.uint8, device="cuda")
    out = torch.empty_like(xd)
    ratios = []
    for e in entries:
        used = ctx.comet_compress(xd, e["eb"], e["nbins"], cont)
        ctx.comet_decompress(cont, used, x.shape, out)
        ctx.comet_sync()
        assert used == _check_layer(oracle, x, e, 64, cont, out)
        ratios.append(x.nbytes / used)
        info = ctx.comet_peek(cont, used)
        assert info.nnz == np.count_nonzero(x)
    assert all(b > a for a, b in zip(ratios, ratios[1:])), ratios     # a looser bound compresses better
    # secondary cells: every error bound with the smallest and with the largest alphabet.  With 1024 bins at a
    # tight bound most residuals are outliers and the container outgrows the input; a cell whose container
    # does not fit the buffer must say so, every other one must match byte for byte and bit for bit
    big = torch.empty(int(comet.comet_compress_bound(x.shape, 1024, 64)), dtype=torch.uint8, device="cuda")
    for e in entries:
        for nb in (1024, 65536):
            if nb == e["nbins"]:
                continue
            cell = dict(e, nbins=nb)
            want = oracle.compress(x, cell["eb"], nb, 64)
            if want.size > cont.numel():
                with pytest.raises(comet.CometError) as ei:
                    ctx.comet_compress(xd, cell["eb"], nb, cont)
                assert ei.value.code == comet.ERR_CAPACITY
            used = ctx.comet_compress(xd, cell["eb"], nb, big)
            assert used == want.size and np.array_equal(big[:used].cpu().numpy(), want), (cell["eb"], nb)
            ctx.comet_decompress(big, used, x.shape, out)
            ctx.comet_sync()
            assert np.array_equal(out.cpu().numpy().ravel().view(np.uint32), oracle.decompress(want).ravel().view(np.uint32)), (cell["eb"], nb)
            _progress(request, f"config 3 cell eb={cell['eb']:.1e} nbins={nb}: ratio {x.nbytes / used:.2f}")
    # adaptive error bound (Sec. 3.2-3.3) fed with seeded synthetic layer statistics and the measured R
    rng = np.random.default_rng(3)
    R = np.count_nonzero(x) / x.size
    for _ in range(16):
        M, L = float(rng.uniform(1e-4, 1e-1)), float(rng.uniform(1e-6, 1e-2))
        got = comet.comet_adapt_eb(M, L, R, 64)
        assert got == oracle.adapt_eb(M, L, R, 64)
        assert got == np.float32(0.01 * M / (0.32 * L * np.sqrt(64 * R)))
    ctx.close()


@pytest.fixture(scope="module")
def config4_oracle(oracle, request):
    """Both tensors of config 4 through the oracle, whole: (input, container, decompressed values) each."""
    entries = synth.config4()

    def one(e):
        x = synth.make(e)
        _progress(request, f"config 4 seed {e['seed']}: input generated")
        want = oracle.compress(x, e["eb"], e["nbins"], 64)
        _progress(request, f"config 4 seed {e['seed']}: oracle container {want.size} bytes")
        want_x = oracle.decompress(want).ravel()
        _progress(request, f"config 4 seed {e['seed']}: oracle decompressed")
        return x, want, want_x

    with ThreadPoolExecutor(max_workers=2) as pool:
        return entries, list(pool.map(one, entries))


def test_config4_two_streams(comet, oracle, config4_oracle, request):
    entries, ref = config4_oracle
    eb, nbins = entries[0]["eb"], entries[0]["nbins"]
    shape = entries[0]["shape"]
    n = int(np.prod(shape))
    ctxs = [comet.Context(max_elems=n, max_nbins=nbins) for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    xs = [torch.from_numpy(r[0]).cuda() for r in ref]
    conts = [torch.zeros(n * 4 // 16 * 16, dtype=torch.uint8, device="cuda") for _ in xs]
    outs = [torch.empty_like(x) for x in xs]
    torch.cuda.synchronize()

    def check(i, what):
        x, want, want_x = ref[i]
        info = ctxs[i].comet_peek(conts[i], conts[i].numel(), stream=streams[i])
        assert int(info.total_bytes) == want.size, f"{what}: size of container {i}"
        assert np.array_equal(conts[i][:want.size].cpu().numpy(), want), f"{what}: container {i} differs from the oracle's"
        assert info.n_active > 2048 and info.nnz == np.count_nonzero(x)
        assert 1.5 < 4.0 * n / want.size < 6.0

    def check_values(i, what):
        x, want, want_x = ref[i]
        got = outs[i].cpu().numpy().ravel()
        assert np.array_equal(got.view(np.uint32), want_x.view(np.uint32)), f"{what}: values of tensor {i} differ from the oracle's"
        assert float((outs[i] - xs[i]).abs().max()) <= float(np.float32(eb))

    # each alone
    for i in range(2):
        ctxs[i].comet_compress(xs[i], eb, nbins, conts[i], stream=streams[i], sync=False)
        ctxs[i].comet_decompress(conts[i], conts[i].numel(), shape, outs[i], stream=streams[i])
        ctxs[i].comet_sync(streams[i])
        check(i, "alone")
        check_values(i, "alone")
        _progress(request, f"config 4 tensor {i} alone: container and values equal the oracle's")

    # overlapped: stream 0 compresses tensor 0 again while stream 1 decompresses tensor 1's container
    outs[1].zero_()
    conts[0].zero_()
    torch.cuda.synchronize()
    ctxs[0].comet_compress(xs[0], eb, nbins, conts[0], stream=streams[0], sync=False)
    ctxs[1].comet_decompress(conts[1], ref[1][1].size, shape, outs[1], stream=streams[1])
    ctxs[0].comet_sync(streams[0])
    ctxs[1].comet_sync(streams[1])
    check(0, "overlapped")
    check_values(1, "overlapped")
    # and the other way round
    outs[0].zero_()
    conts[1].zero_()
    torch.cuda.synchronize()
    ctxs[1].comet_compress(xs[1], eb, nbins, conts[1], stream=streams[1], sync=False)
    ctxs[0].comet_decompress(conts[0], ref[0][1].size, shape, outs[0], stream=streams[0])
    ctxs[0].comet_sync(streams[0])
    ctxs[1].comet_sync(streams[1])
    check(1, "overlapped")
    check_values(0, "overlapped")
    for c in ctxs:
        c.close()
