"""q8_linear_f32_static -- the entry point for callers that cannot allocate -- against q8_linear_f32, through the
C ABI: same bytes out (fp32 outputs, int8 codes under the requantize epilogue, abs-max, scale), on two calls in
a row that share the library's static scratch, the second with a smaller input than the first; then the size
limit.  Runs last (the file name sorts after the other tests) and also on its own in a fresh process."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_1910_06188_amd import synth  # noqa: E402


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1910_06188_amd import q8 as mod
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(q8, lib, M, K, N, seed, flags, n_groups=1):
    """The existing entry point and the static one on the same inputs, raw C ABI; returns what each wrote."""
    g = synth.rng(seed)
    x = dev(synth.activations(g, M, K))
    wq = dev(synth.random_int8(g, (N, K)))
    b = dev(synth.bias(g, N))
    sw = dev(np.linspace(900.0, 1400.0, n_groups).astype(np.float32))
    ns = torch.tensor([127.0 / 6.0], device="cuda")
    out_dtype = torch.int8 if flags & q8.EPI_REQUANT else torch.float32
    st = torch.cuda.current_stream().cuda_stream
    res = []
    for static in (False, True):
        y = torch.full((M, N), 7, dtype=out_dtype, device="cuda")
        amax = torch.full((1,), 1e9, device="cuda")
        stats = torch.full((2,), -1.0, device="cuda")
        if static:
            rc = lib.q8_linear_f32_static(x.data_ptr(), wq.data_ptr(), b.data_ptr(), sw.data_ptr(), n_groups, M, N, K,
                                          y.data_ptr(), stats.data_ptr(), amax.data_ptr(), ns.data_ptr(), flags, st)
        else:
            xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
            scal = torch.zeros(q8.SCAL_WORK, device="cuda")
            rc = lib.q8_linear_f32(x.data_ptr(), wq.data_ptr(), b.data_ptr(), sw.data_ptr(), n_groups, M, N, K,
                                   xq.data_ptr(), scal.data_ptr(), y.data_ptr(), None, amax.data_ptr(), ns.data_ptr(),
                                   flags, st)
            stats = scal[:2].clone()
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        res.append((y.cpu().numpy(), amax.cpu().numpy(), stats.cpu().numpy()))
    return res


def test_static_scratch_entry_point_matches_linear_f32(q8):
    lib = q8.raw()
    # two calls in a row on the shared scratch, the second smaller; then more shapes and epilogues, the
    # single-workgroup quantizer (M*K <= 16384) and a ragged shape on the generic GEMM included
    cases = [(1536, 1024, 768, q8.EPI_GELU | q8.EPI_ABSMAX, 1), (300, 256, 520, q8.EPI_GELU | q8.EPI_ABSMAX, 1),
             (700, 384, 600, 0, 3), (16, 768, 768, q8.EPI_ABSMAX, 1), (512, 1024, 1024, q8.EPI_GELU | q8.EPI_REQUANT, 1),
             (33, 100, 70, 0, 1), (4096, 4096, 256, 0, 1), (5, 128, 128, q8.EPI_REQUANT, 1)]
    for i, (M, K, N, flags, n_groups) in enumerate(cases):
        (y0, a0, s0), (y1, a1, s1) = both(q8, lib, M, K, N, 9100 + i, flags, n_groups)
        assert np.array_equal(y0, y1), (M, K, N, flags)
        assert np.array_equal(s0, s1) and s1[0] > 0 and s1[1] == np.float32(127.0) / s1[0], (M, K, N, flags)
        if flags & q8.EPI_ABSMAX:
            assert a0[0] == a1[0] == np.abs(y1).max()
    # an empty activation tensor: nothing to quantize, nothing written
    p = 0x1000
    assert lib.q8_linear_f32_static(None, None, None, p, 1, 0, 8, 128, None, None, None, None, 0, None) == 0
    # beyond the static scratch: refused on the host, nothing launched
    lim = q8.STATIC_MAX_CODES
    assert lib.q8_linear_f32_static(p, p, None, p, 1, lim // 1024 + 1, 8, 1024, p, None, None, None, 0, None) == 6
    assert lib.q8_linear_f32_static(p, p, None, p, 1, 1 << 40, 8, 128, p, None, None, None, 0, None) == 6
    assert b"static scratch" in C.cast(lib.q8_status_str(6), C.c_char_p).value
    torch.cuda.synchronize()
