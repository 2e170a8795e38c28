"""Parity at the benchmark's full shapes (the four FC GEMMs of the BERT-Large encoder layer at
12288 tokens, and the BERT-Base ones), in the launch configuration bench.py times (automatic
tile choice).  Every stage is compared in full: all int8 codes, every int32 accumulator and
every fp32 output against the oracle (its integer GEMM runs threaded over rows, which does
not change an exact result)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import q8_oracle as O  # noqa: E402
from paper_1910_06188_amd import synth  # noqa: E402


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1910_06188_amd import q8 as mod
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def one():
    return torch.zeros(1, device="cuda")


@pytest.mark.parametrize("M,K,N,gelu", [(12288, 1024, 4096, True), (12288, 4096, 1024, False),
                                        (12288, 1024, 3072, False), (12288, 1024, 1024, False),
                                        (4096, 768, 3072, False), (4096, 3072, 768, False),
                                        (4096, 768, 768, False), (8192, 768, 2304, False)])
def test_fullsize_fc_whole_output(q8, M, K, N, gelu):
    g = synth.rng(7000 + N)
    x = synth.activations(g, M, K)
    n_groups = 3 if N in (3072, 2304) and K in (1024, 768) and not gelu else 1
    Ws = [synth.weights(g, N // n_groups, K) * np.float32(1.0 + 0.5 * i) for i in range(n_groups)]
    b = synth.bias(g, N)
    # weights offline on the GPU, checked against the oracle in full
    wqs, sws = [], []
    for W in Ws:
        wd = dev(W)
        a, s = one(), one()
        q8.q8_absmax(wd, a, s)
        wq = torch.empty(W.shape, dtype=torch.int8, device="cuda")
        q8.q8_quantize(wd, s, wq)
        wq_ref, s_ref = O.quantize_tensor(W)
        assert s.item() == float(s_ref)
        np.testing.assert_array_equal(wq.cpu().numpy(), wq_ref)
        wqs.append(wq)
        sws.append(s)
    wq = torch.cat(wqs, 0).contiguous()
    sw = torch.cat(sws).contiguous()
    # activations: abs-max, scale and every int8 code against the oracle
    xd = dev(x)
    a, sx = one(), one()
    q8.q8_absmax(xd, a, sx)
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    q8.q8_quantize(xd, sx, xq)
    sx_ref = O.scale(O.absmax(x))
    assert a.item() == float(O.absmax(x)) and sx.item() == float(sx_ref)
    xq_ref = O.quantize(x, sx_ref)
    np.testing.assert_array_equal(xq.cpu().numpy(), xq_ref)
    # GEMM + epilogue
    y = torch.empty((M, N), device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    amax = one()
    flags = (q8.EPI_GELU | q8.EPI_ABSMAX) if gelu else 0
    q8.q8_linear(xq, wq, dev(b), sx, sw, y, n_groups=n_groups, acc_out=acc, out_amax=amax if gelu else None,
                 flags=flags)
    y_plain = None
    if not gelu:
        y_plain = torch.empty((M, N), device="cuda")
        q8.q8_linear(xq, wq, dev(b), sx, sw, y_plain, n_groups=n_groups)      # the kernel bench.py times
    torch.cuda.synchronize()
    swh = sw.cpu().numpy()
    bq = O.quantize_bias(b, N, sx_ref, swh)
    acc_ref = O.gemm_i8(xq_ref, wq.cpu().numpy(), bq, threads=16)          # the whole [M, N] accumulator
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_ref)
    y_ref = O.dequant(acc_ref, sx_ref, swh)
    yh = y.cpu().numpy()
    if gelu:
        gl = O.gelu(y_ref).astype(np.float64)
        assert np.all(np.abs(yh.astype(np.float64) - gl) <= 1e-6 + 1e-5 * np.abs(gl))
        assert amax.item() == np.abs(yh).max()
        # the kernel bench.py times (no accumulator dump) writes the same bytes
        y2, amax2 = torch.empty((M, N), device="cuda"), one()
        q8.q8_linear(xq, wq, dev(b), sx, sw, y2, n_groups=n_groups, out_amax=amax2, flags=flags)
        assert torch.equal(y, y2) and amax2.item() == amax.item()
    else:
        ref64 = y_ref.astype(np.float64)
        assert np.all(np.abs(yh.astype(np.float64) - ref64) <= 1e-6 * np.abs(ref64))
        # the two kernels (with and without the accumulator dump) agree everywhere
        assert torch.equal(y, y_plain)


def test_fullsize_embedding_bert_base_tables(q8):
    tabs = synth.embedding_tables(seed=5, hidden=768)
    ids = synth.token_ids(seed=6, batch=64, seq=128)
    qs = {k: O.quantize_tensor(v) for k, v in tabs.items()}
    order = ("word", "position", "token_type")
    out = torch.empty((64 * 128, 768), device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    scales = dev(np.array([qs[k][1] for k in order], np.float32))
    q8.q8_embedding_sum3(*[dev(qs[k][0]) for k in order], scales, *[dev(ids[k]) for k in order], out, err_flag=flag)
    ref = O.embedding_sum3(qs["word"][0], qs["word"][1], qs["position"][0], qs["position"][1],
                           qs["token_type"][0], qs["token_type"][1], ids["word"], ids["position"], ids["token_type"])
    mag = sum(np.abs(qs[k][0][ids[k]].astype(np.float64)) / float(qs[k][1]) for k in order)
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - ref) <= 1e-6 * mag + 1e-12)
    assert flag.item() == 0
    # single-table int8 gather, full word table
    o8 = torch.empty((64 * 128, 768), dtype=torch.int8, device="cuda")
    q8.q8_embedding(dev(qs["word"][0]), scales[0:1], dev(ids["word"]), o8)
    np.testing.assert_array_equal(o8.cpu().numpy(), qs["word"][0][ids["word"]])


def test_output_beyond_2_gib(q8):
    """y and the accumulator dump larger than 2^31 bytes each (140000 x 4096 fp32 = 2.29 GB): the MFMA
    kernel addresses its stores from each tile's first row, so the size of y does not matter.  Rows on both
    sides of the 2^31-byte boundary, the first, the last full tile and the ragged last rows are compared
    with the oracle; every tile shape."""
    M, N, K = 140000, 4096, 128
    g = synth.rng(77)
    xq = synth.random_int8(g, (M, K))
    wq = synth.random_int8(g, (N, K))
    b = synth.bias(g, N)
    sx, sw = np.float32(31.5), np.float32(1270.0)
    rows = np.array([0, 1, 191, 192, 131071, 131072, 131073, 139775, 139776, 139999])     # 2^31 / (4096*4) = 131072
    bq = O.quantize_bias(b, N, sx, np.array([sw], np.float32))
    acc_ref = O.gemm_i8(xq[rows], wq, bq)
    y_ref = O.dequant(acc_ref, sx, np.array([sw], np.float32))
    xd, wd, bd = dev(xq), dev(wq), dev(b)
    sxd, swd = torch.tensor([float(sx)], device="cuda"), torch.tensor([float(sw)], device="cuda")
    y = torch.empty((M, N), device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    ridx = torch.from_numpy(rows).cuda()
    for variant in (0, 2, 3, 5, 6):
        q8.set_gemm_variant(variant)
        try:
            y.zero_()
            q8.q8_linear(xd, wd, bd, sxd, swd, y)                      # specialised kernel
            got = y[ridx].cpu().numpy()
            assert np.all(np.abs(got.astype(np.float64) - y_ref) <= 1e-6 * np.abs(y_ref.astype(np.float64))), variant
            y.zero_()
            q8.q8_linear(xd, wd, bd, sxd, swd, y, acc_out=acc)          # run-time-flag kernel with the dump
            np.testing.assert_array_equal(acc[ridx].cpu().numpy(), acc_ref, err_msg=f"variant {variant}")
            np.testing.assert_array_equal(y[ridx].cpu().numpy(), got)
        finally:
            q8.set_gemm_variant(0)


def test_operand_beyond_2_gib(q8):
    """An activation tensor larger than 2^31 bytes (524388 x 4096 int8 codes): the MFMA kernel addresses its
    operand loads from each tile's first row as well.  Rows around the 2^31-byte boundary and the ragged
    end against the oracle."""
    M, N, K = 524388, 256, 4096
    g = synth.rng(78)
    xq = synth.random_int8(g, (M, K))
    wq = synth.random_int8(g, (N, K))
    b = synth.bias(g, N)
    sx, sw = np.float32(31.5), np.float32(1270.0)
    rows = np.array([0, 255, 256, 524287, 524288, 524289, 524387])          # 2^31 / 4096 = 524288
    bq = O.quantize_bias(b, N, sx, np.array([sw], np.float32))
    acc_ref = O.gemm_i8(xq[rows], wq, bq)
    y_ref = O.dequant(acc_ref, sx, np.array([sw], np.float32))
    xd, wd, bd = dev(xq), dev(wq), dev(b)
    sxd, swd = torch.tensor([float(sx)], device="cuda"), torch.tensor([float(sw)], device="cuda")
    y = torch.empty((M, N), device="cuda")
    ridx = torch.from_numpy(rows).cuda()
    for variant in (0, 3, 5):
        q8.set_gemm_variant(variant)
        try:
            y.zero_()
            q8.q8_linear(xd, wd, bd, sxd, swd, y)
            got = y[ridx].cpu().numpy()
            assert np.all(np.abs(got.astype(np.float64) - y_ref) <= 1e-6 * np.abs(y_ref.astype(np.float64))), variant
        finally:
            q8.set_gemm_variant(0)


def test_elementwise_beyond_2_31_elements(q8):
    """abs-max and quantize on 2^31 + 4099 floats (8.6 GB): element indices do not fit 32 bits.  The
    extreme value sits past the 2^31-th element; every code is compared with the oracle."""
    n = (1 << 31) + 4099
    g = synth.rng(79)
    block = g.standard_normal(1 << 24, dtype=np.float32)
    x = np.tile(block, (n + block.size - 1) // block.size)[:n]
    x[n - 7] = np.float32(-9.75)                                  # the abs-max, beyond index 2^31
    x[(1 << 31) + 1] = np.float32(9.5)
    xd = torch.from_numpy(x).cuda()
    amax, sc = one(), one()
    q8.q8_absmax(xd, amax, sc)
    assert amax.item() == 9.75 and sc.item() == float(O.scale(np.float32(9.75)))
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    q8.q8_quantize(xd, sc, q)
    qh = q.cpu().numpy()
    ref = O.quantize(x, O.scale(np.float32(9.75)))
    assert qh[n - 7] == -127 and np.array_equal(qh, ref)
    # the fused form (partial maxima folded by the quantize kernel) on the same tensor
    scal = torch.zeros(q8.SCAL_WORK, device="cuda")
    q.zero_()
    y = torch.empty((1, 1), device="cuda")
    w1 = torch.ones((1, 1), dtype=torch.int8, device="cuda")
    lib = q8.raw()
    rc = lib.q8_linear_f32(xd.data_ptr(), w1.data_ptr(), None, sc.data_ptr(), 1, n, 1, 1, q.data_ptr(), scal.data_ptr(),
                           torch.empty((n, 1), device="cuda").data_ptr(), None, None, None, 0, None)
    assert rc == 0
    torch.cuda.synchronize()
    assert scal[0].item() == 9.75 and np.array_equal(q.cpu().numpy(), ref)
