"""comet_decompress_static: decompression without a context and without any allocation, from the
library's static scratch array.  Its output must equal comet_decompress's bit for bit (and the
oracle's), on two calls in a row, the second with a smaller input, so that nothing the first call left
in the array leaks into the second.
"""
import ctypes as C

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


def _container(oracle, x, eb, nbins, chunk):
    buf = oracle.compress(x, eb, nbins, chunk)
    pad = np.zeros((-buf.size) % 16, np.uint8)
    return buf, torch.from_numpy(np.concatenate([buf, pad])).cuda()


def test_static_decompress_equals_context_decompress(comet, oracle):
    cases = [((4, 16, 56, 56), 1e-2, 1024, 64),        # 200 704 elements
             ((2, 3, 37, 33), 1e-3, 1024, 64),         # smaller, odd width, ragged last chunk
             ((1, 2, 9, 600), 1e-2, 4096, 128),        # planes wider than 512 columns: the other kernel
             ((3, 40, 7, 7), 5e-2, 64, 64)]            # small planes, escapes
    ctx = comet.Context(max_elems=max(int(np.prod(c[0])) for c in cases), max_nbins=4096)
    status = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    for shape, eb, nbins, chunk in cases:
        x = synth.relu_blur(shape, seed=int(np.prod(shape)) % 1000, blur=3, shift=-0.2)
        x.ravel()[3] = np.inf
        x.ravel()[x.size // 2] = -7.5e8                 # verbatim values
        buf, cont = _container(oracle, x, eb, nbins, chunk)
        ref = torch.empty(x.size, dtype=torch.float32, device="cuda")
        ctx.comet_decompress(cont, buf.size, shape, ref)
        ctx.comet_sync()
        out = torch.full((x.size,), -1.0, dtype=torch.float32, device="cuda")
        comet.comet_decompress_static(cont, buf.size, shape, out, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32)), shape
        assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.decompress(buf).ravel().view(np.uint32)), shape
    ctx.close()


def test_static_decompress_errors(comet, oracle):
    shape = (1, 4, 28, 28)
    x = synth.relu_blur(shape, seed=9)
    buf, cont = _container(oracle, x, 1e-2, 1024, 64)
    out = torch.zeros(x.size, dtype=torch.float32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    # a tensor beyond the static work buffer is refused before any launch
    big = (1, 1, 2049, 2048)
    assert int(np.prod(big)) > comet.STATIC_MAX_ELEMS
    with pytest.raises(comet.CometError) as ei:
        comet.comet_decompress_static(cont, buf.size, big, out, status)
    assert ei.value.code == comet.ERR_NOMEM
    with pytest.raises(comet.CometError) as ei:
        comet.comet_decompress_static(cont, buf.size, (0, 1, 1, 1), out, status)
    assert ei.value.code == comet.ERR_INVALID
    # a malformed container is reported through the status word, and the next call is clean
    bad = cont.clone()
    bad[0] = 0x58
    comet.comet_decompress_static(bad, buf.size, shape, out, status)
    torch.cuda.synchronize()
    assert int(status.item()) == comet.ERR_FORMAT
    comet.comet_decompress_static(cont, buf.size, shape, out, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.decompress(buf).ravel().view(np.uint32))
    comet.comet_decompress_static(cont, buf.size, shape, out, None)            # the status word is optional
    torch.cuda.synchronize()
