"""GPU parity: every entry point of the C ABI against the CPU oracle on the same
seeded inputs.  int8 codes and int32 accumulators must match bit for bit; fp32
outputs within 1e-6 relative (the accumulator is an exact integer, so the relative
error of the dequantised value does not depend on magnitude)."""
import json
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import q8_oracle as O  # noqa: E402
from paper_1910_06188_amd import synth  # noqa: E402

RTOL = 1e-6          # fp32 dequantised outputs
GELU_RTOL, GELU_ATOL = 1e-5, 1e-6   # fp32 erfc on the GPU vs fp64 on the host


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1910_06188_amd import q8 as mod
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def scalar(v, dtype=torch.float32):
    return torch.tensor([v], dtype=dtype, device="cuda")


def assert_rel(got, ref, rtol=RTOL, atol=0.0):
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    err = np.abs(got - ref)
    tol = atol + rtol * np.abs(ref)
    bad = err > tol
    assert not bad.any(), f"{bad.sum()} of {bad.size} outside tolerance; worst rel {np.max(err / np.maximum(np.abs(ref), 1e-30)):.3e}"


# --------------------------------------------------------------------------- abs-max / scale
@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 63, 64, 255, 1023, 4096, 4099, 1_000_003, 12_582_912])
def test_absmax_and_scale(q8, n):
    g = synth.rng(100 + n % 97)
    x = g.standard_normal(n, dtype=np.float32) * np.float32(2.5)
    if n > 10:
        x[g.integers(0, n)] = np.float32(-77.25)      # a negative extreme somewhere
    xd = dev(x)
    amax = torch.full((1,), -1.0, device="cuda")
    sc = torch.full((1,), -1.0, device="cuda")
    q8.q8_absmax(xd, amax, sc)
    a_ref = O.absmax(x)
    assert host(amax)[0] == a_ref
    assert host(sc)[0] == O.scale(a_ref)
    # scale optional
    amax2 = torch.full((1,), -1.0, device="cuda")
    q8.q8_absmax(xd, amax2, None)
    assert host(amax2)[0] == a_ref


def test_absmax_misaligned_views_and_tail_positions(q8):
    g = synth.rng(7)
    base = g.standard_normal(5000, dtype=np.float32)
    bd = dev(base)
    for off in (1, 2, 3):
        for n in (1, 2, 7, 1000, 4993):
            x = base[off:off + n]
            amax, sc = scalar(0.0), scalar(0.0)
            q8.q8_absmax(bd[off:off + n], amax, sc)
            assert host(amax)[0] == O.absmax(x)
    # the extreme placed at every position near the vector head/tail boundaries
    n = 1030
    for pos in list(range(0, 9)) + list(range(n - 9, n)):
        x = np.full(n, 0.5, np.float32)
        x[pos] = -3.0
        amax = scalar(0.0)
        q8.q8_absmax(dev(x)[0:n], amax, None)
        assert host(amax)[0] == 3.0
    # all zeros: S = 1
    amax, sc = scalar(-1.0), scalar(-1.0)
    q8.q8_absmax(torch.zeros(1000, device="cuda"), amax, sc)
    assert host(amax)[0] == 0.0 and host(sc)[0] == 1.0


def test_scale_from_amax(q8):
    for a in (0.0, 1.0, 5.2173, 127.0, 0.0999, 3e-30):
        out = scalar(-1.0)
        q8.q8_scale_from_amax(scalar(a), out)
        assert host(out)[0] == O.scale(np.float32(a))


# --------------------------------------------------------------------------- quantize
def test_quantize_hand_cases(q8, golden_dir):
    with open(os.path.join(golden_dir, "quantize_cases.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        x = np.array(c["x"], dtype=np.float32)
        xd = dev(x)
        sc = scalar(float(c["scale"]))
        if c["dynamic"]:
            amax = scalar(0.0)
            q8.q8_absmax(xd, amax, sc)
            assert host(amax)[0] == np.float32(c["amax"]) and host(sc)[0] == np.float32(c["scale"])
        q = torch.zeros(x.size, dtype=torch.int8, device="cuda")
        q8.q8_quantize(xd, sc, q)
        assert host(q).tolist() == c["q"], c["name"]


@pytest.mark.parametrize("n", [1, 2, 3, 5, 1024, 4097, 999_999, 3_145_728])
def test_quantize_bit_exact_dynamic(q8, n):
    g = synth.rng(200 + n % 89)
    x = g.standard_normal(n, dtype=np.float32)
    xd = dev(x)
    amax, sc = scalar(0.0), scalar(0.0)
    q = torch.empty(n, dtype=torch.int8, device="cuda")
    q8.q8_absmax(xd, amax, sc)
    q8.q8_quantize(xd, sc, q)
    s = O.scale(O.absmax(x))
    assert host(sc)[0] == s
    np.testing.assert_array_equal(host(q), O.quantize(x, s))


def test_quantize_ties_static_scales_and_misalignment(q8):
    g = synth.rng(31)
    for s in (1.0, 0.5, 63.5, 24.413, 1270.5, 0.037):
        s32 = np.float32(s)
        ties = (np.arange(-140, 141, dtype=np.float32) + np.float32(0.5)) / s32
        x = np.concatenate([ties, np.nextafter(ties, np.float32(np.inf)), np.nextafter(ties, np.float32(-np.inf)),
                            g.standard_normal(5000, dtype=np.float32) * np.float32(100 / s),
                            np.array([1e10, -1e10, 0.0, -0.0, 1e-40, -1e-40], dtype=np.float32)]).astype(np.float32)
        xd = dev(x)
        for off in (0, 1, 2, 3):
            n = x.size - off - 5
            qbuf = torch.zeros(x.size + 8, dtype=torch.int8, device="cuda")
            for qoff in (0, 1):
                q = qbuf[qoff:qoff + n]
                q8.q8_quantize(xd[off:off + n], scalar(float(s32)), q)
                np.testing.assert_array_equal(host(q), O.quantize(x[off:off + n], s32))
    # writes stay inside q
    qbuf = torch.full((64,), 99, dtype=torch.int8, device="cuda")
    q8.q8_quantize(dev(np.ones(13, np.float32)), scalar(5.0), qbuf[8:21])
    hb = host(qbuf)
    assert np.all(hb[:8] == 99) and np.all(hb[21:] == 99) and np.all(hb[8:21] == 5)


# --------------------------------------------------------------------------- linear
def run_linear(q8, x, W, b, n_groups=1, flags=0, sx_static=None, next_scale=None, variant=0, Ws=None):
    """GPU chain absmax -> quantize -> linear through the C ABI; returns host arrays."""
    M, K = x.shape
    if Ws is None:
        Ws = [W]
    wq_parts, sw_parts = [], []
    for Wp in Ws:                              # weights: same kernels, offline (Eq. 3 + Eq. 1)
        wd = dev(Wp)
        a, s = scalar(0.0), scalar(0.0)
        q8.q8_absmax(wd, a, s)
        wq = torch.empty(Wp.shape, dtype=torch.int8, device="cuda")
        q8.q8_quantize(wd, s, wq)
        wq_parts.append(wq)
        sw_parts.append(s)
    wq = torch.cat(wq_parts, 0).contiguous()
    sw = torch.cat(sw_parts).contiguous()
    N = wq.shape[0]
    xd = dev(x)
    amax, sx = scalar(0.0), scalar(0.0)
    if sx_static is None:
        q8.q8_absmax(xd, amax, sx)
    else:
        sx = scalar(float(sx_static))
    xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
    q8.q8_quantize(xd, sx, xq)
    y = torch.empty((M, N), dtype=torch.int8 if flags & 4 else torch.float32, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    out_amax = scalar(0.0)
    ns = None if next_scale is None else scalar(float(next_scale))
    q8.set_gemm_variant(variant)
    try:
        q8.q8_linear(xq, wq, None if b is None else dev(b), sx, sw, y, n_groups=n_groups, acc_out=acc,
                     out_amax=out_amax if flags & 2 else None, next_scale=ns, flags=flags)
        y2 = None
        if flags == 0:                                    # the dedicated fp32-only kernel as well
            y2 = torch.empty((M, N), dtype=torch.float32, device="cuda")
            q8.q8_linear(xq, wq, None if b is None else dev(b), sx, sw, y2, n_groups=n_groups)
    finally:
        q8.set_gemm_variant(0)
    torch.cuda.synchronize()
    return dict(xq=host(xq), wq=host(wq), sw=host(sw), sx=host(sx)[0], acc=host(acc), y=host(y),
                y_plain=None if y2 is None else host(y2), out_amax=host(out_amax)[0])


def check_linear(r, x, b, act_gelu=False, sx_static=None, threads=8):
    """Oracle on the same inputs; weights' codes are checked against the oracle too."""
    ref = O.linear(x, r["wq"], r["sw"], b, sx=sx_static, act_gelu=False, threads=threads)
    assert r["sx"] == ref["sx"]
    np.testing.assert_array_equal(r["xq"], ref["xq"])
    np.testing.assert_array_equal(r["acc"], ref["acc"])
    return ref


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6])
def test_linear_single_fc_config(q8, variant):
    d = synth.single_fc(0)                                  # 16 x 768 -> 768
    r = run_linear(q8, d["x"], d["W"], d["b"], variant=variant)
    wq_ref, sw_ref = O.quantize_tensor(d["W"])
    np.testing.assert_array_equal(r["wq"], wq_ref)
    assert r["sw"][0] == sw_ref
    ref = check_linear(r, d["x"], d["b"])
    assert_rel(r["y"], ref["y"])
    assert_rel(r["y_plain"], ref["y"])


@pytest.mark.parametrize("M,K,N,variant", [
    (300, 256, 520, 0), (700, 384, 600, 1), (700, 384, 600, 2), (700, 384, 600, 3), (700, 384, 600, 4),
    (257, 128, 129, 1), (1, 128, 1, 3), (513, 1024, 257, 2), (255, 640, 1000, 4), (1030, 256, 2100, 1), (768, 384, 512, 4), (512, 1024, 512, 2),
    (700, 384, 600, 5), (385, 256, 770, 5), (768, 1024, 512, 5), (700, 384, 600, 6), (385, 256, 770, 6), (768, 1024, 512, 6),
    # the launcher's own choice (variant 0) on every shape class above: short and long K, ragged and exact edges,
    # fewer tiles than compute units and several rounds of them
    (700, 384, 600, 0), (257, 128, 129, 0), (1, 128, 1, 0), (513, 1024, 257, 0), (255, 640, 1000, 0), (1030, 256, 2100, 0),
    (768, 384, 512, 0), (512, 1024, 512, 0), (385, 256, 770, 0), (768, 1024, 512, 0), (520, 2048, 300, 0), (3000, 4096, 260, 0),
    (4100, 512, 3000, 0),
])
def test_linear_mfma_ragged_multi_tile(q8, M, K, N, variant):
    d = synth.fc_layer(1000 + M + N, M, K, N)
    r = run_linear(q8, d["x"], d["W"], d["b"], variant=variant)
    ref = check_linear(r, d["x"], d["b"])
    assert_rel(r["y"], ref["y"])
    assert_rel(r["y_plain"], ref["y"])


@pytest.mark.parametrize("M,K,N", [(33, 100, 70), (5, 1, 3), (64, 127, 64), (17, 200, 19), (2, 3000, 2), (40, 0, 8)])
def test_linear_generic_path_any_shape(q8, M, K, N):
    d = synth.fc_layer(2000 + M + K, M, max(K, 1), N)
    x = d["x"][:, :K]
    W = d["W"][:, :K]
    if K == 0:                                              # no reduction: y is the dequantised bias
        xq = torch.empty((M, 0), dtype=torch.int8, device="cuda")
        wq = torch.empty((N, 0), dtype=torch.int8, device="cuda")
        y = torch.empty((M, N), device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        q8.q8_linear(xq, wq, dev(d["b"]), scalar(2.0), scalar(8.0), y, acc_out=acc)
        bq = O.quantize_bias(d["b"], N, 2.0, [8.0])
        np.testing.assert_array_equal(host(acc), np.broadcast_to(bq, (M, N)))
        assert_rel(host(y), O.dequant(np.broadcast_to(bq, (M, N)).copy(), 2.0, [8.0]))
        return
    r = run_linear(q8, x, W, d["b"])
    ref = check_linear(r, x, d["b"])
    assert_rel(r["y"], ref["y"])
    assert_rel(r["y_plain"], ref["y"])


def test_linear_misaligned_operands_take_generic_path(q8):
    g = synth.rng(41)
    M, K, N = 20, 256, 24
    xq = synth.random_int8(g, (M, K))
    wq = synth.random_int8(g, (N, K))
    buf_x = torch.zeros(M * K + 16, dtype=torch.int8, device="cuda")
    buf_x[1:1 + M * K] = dev(xq).reshape(-1)
    xv = buf_x[1:1 + M * K].view(M, K)
    y = torch.empty((M, N), device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    q8.q8_linear(xv, dev(wq), None, scalar(3.0), scalar(7.0), y, acc_out=acc)
    np.testing.assert_array_equal(host(acc), O.gemm_i8(xq, wq))


def test_linear_no_bias_and_grouped_qkv(q8):
    g = synth.rng(42)
    M, K, H = 200, 256, 128
    x = synth.activations(g, M, K)
    Ws = [synth.weights(g, H, K) * np.float32(f) for f in (1.0, 2.5, 0.3)]
    b = np.concatenate([synth.bias(g, H) for _ in range(3)])
    r = run_linear(q8, x, None, b, n_groups=3, Ws=Ws)
    ref = check_linear(r, x, b)
    assert_rel(r["y"], ref["y"])
    assert len(set(r["sw"].tolist())) == 3
    r0 = run_linear(q8, x, Ws[0], None)
    ref0 = check_linear(r0, x, None)
    assert_rel(r0["y"], ref0["y"])


def test_linear_int32_exactness_stress(q8):
    """Sums that are odd and far above 2^24: any floating-point accumulation would miss them."""
    K = 4096
    for M, N in ((3, 2), (130, 260)):
        xq = np.full((M, K), 127, np.int8)
        wq = np.full((N, K), -127, np.int8)
        wq[:, 0] = -126                                     # makes the sum odd: -(4095*16129 + 127*126)
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y = torch.empty((M, N), device="cuda")
        q8.q8_linear(dev(xq), dev(wq), None, scalar(1.0), scalar(1.0), y, acc_out=acc)
        assert np.all(host(acc) == -(4095 * 16129 + 127 * 126))
        assert_rel(host(y), O.dequant(host(acc), 1.0, [1.0]))
    # extreme codes incl. -128 at the largest K the MFMA path takes
    K = 131072 - 128
    xq = np.full((2, K), -128, np.int8)
    wq = np.full((2, K), -128, np.int8)
    acc = torch.empty((2, 2), dtype=torch.int32, device="cuda")
    y = torch.empty((2, 2), device="cuda")
    q8.q8_linear(dev(xq), dev(wq), None, scalar(1.0), scalar(1.0), y, acc_out=acc)
    assert np.all(host(acc) == 16384 * K)
    # alternating signs cancel exactly
    K = 1024
    alt = np.where(np.arange(K) % 2 == 0, 127, -127).astype(np.int8)
    acc = torch.empty((1, 1), dtype=torch.int32, device="cuda")
    q8.q8_linear(dev(alt[None, :]), dev(np.full((1, K), 127, np.int8)), None, scalar(1.0), scalar(1.0),
                 torch.empty((1, 1), device="cuda"), acc_out=acc)
    assert host(acc)[0, 0] == 0


def test_linear_random_int8_all_variants_asymmetric(q8):
    """Raw int8 operands (no quantize step): pins the MFMA operand and accumulator layout."""
    g = synth.rng(43)
    M, K, N = 290, 384, 410
    xq = synth.random_int8(g, (M, K), -128, 127)
    wq = synth.random_int8(g, (N, K), -128, 127)
    ref = O.gemm_i8(xq, wq, threads=8)
    for variant in (1, 2, 3, 4, 5, 6):
        q8.set_gemm_variant(variant)
        try:
            acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
            q8.q8_linear(dev(xq), dev(wq), None, scalar(1.0), scalar(1.0), torch.empty((M, N), device="cuda"),
                         acc_out=acc)
        finally:
            q8.set_gemm_variant(0)
        np.testing.assert_array_equal(host(acc), ref, err_msg=f"variant {variant}")


def test_linear_random_shapes_every_variant(q8):
    """Seeded random shapes (ragged in every dimension, K on and off the MFMA grid) through every tile
    variant, with and without bias, one or three weight-scale groups: the whole dynamic chain against the
    oracle, plus the dedicated fp32 kernel against the run-time-flag one."""
    g = synth.rng(2024)
    for case in range(28):
        M = int(g.integers(1, 700))
        K = int(g.choice([128, 256, 384, 512, 640])) if case % 4 else int(g.integers(1, 300))
        n_groups = 3 if case % 3 == 0 else 1
        N = int(g.integers(1, 260)) * n_groups
        variant = case % 7
        d = synth.fc_layer(3000 + case, M, K, N)
        Ws = [d["W"][i * (N // n_groups):(i + 1) * (N // n_groups)] * np.float32(1 + 0.5 * i) for i in range(n_groups)]
        b = d["b"] if case % 5 else None
        r = run_linear(q8, d["x"], None, b, n_groups=n_groups, variant=variant, Ws=Ws)
        ref = check_linear(r, d["x"], b)
        assert_rel(r["y"], ref["y"])
        np.testing.assert_array_equal(r["y_plain"], r["y"], err_msg=f"case {case}: M={M} K={K} N={N} variant={variant}")


def test_linear_bias_saturation(q8):
    with open(os.path.join(os.path.dirname(__file__), "golden", "bias_cases.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        b = np.array(c["b"], np.float32)
        N = b.size
        K = 128
        acc = torch.empty((1, N), dtype=torch.int32, device="cuda")
        q8.q8_linear(torch.zeros((1, K), dtype=torch.int8, device="cuda"),
                     torch.zeros((N, K), dtype=torch.int8, device="cuda"), dev(b), scalar(c["sx"]),
                     dev(np.array(c["sw"], np.float32)), torch.empty((1, N), device="cuda"),
                     n_groups=len(c["sw"]), acc_out=acc)
        assert host(acc)[0].tolist() == c["bq"], c["name"]


def test_linear_zero_input_tensor(q8):
    d = synth.fc_layer(44, 130, 256, 140)
    x = np.zeros_like(d["x"])
    r = run_linear(q8, x, d["W"], d["b"])
    assert r["sx"] == 1.0 and not r["xq"].any()
    ref = check_linear(r, x, d["b"])
    assert_rel(r["y"], ref["y"])


@pytest.mark.parametrize("M,K,N", [(300, 256, 520), (33, 100, 70)])
def test_linear_epilogue_gelu_absmax_requant(q8, M, K, N):
    d = synth.fc_layer(45 + M, M, K, N)
    x, W, b = d["x"], d["W"] * np.float32(8.0), d["b"]
    # GELU + abs-max, fp32 out
    r = run_linear(q8, x, W, b, flags=1 | 2)
    ref = check_linear(r, x, b)
    gl = O.gelu(ref["y"])
    assert_rel(r["y"], gl, rtol=GELU_RTOL, atol=GELU_ATOL)
    assert r["out_amax"] == np.abs(r["y"]).max()           # abs-max of the values the GPU itself wrote
    # abs-max alone on the plain dequantised output
    r2 = run_linear(q8, x, W, b, flags=2)
    ref2 = check_linear(r2, x, b)
    assert_rel(r2["y"], ref2["y"])
    assert r2["out_amax"] == np.abs(r2["y"]).max()
    # requantise with a stored scale: codes from the GPU's own fp32 values (stage-wise rule);
    # against the oracle's fp32 values they may differ by one code only where the product
    # sits within rounding distance of a tie
    ns = np.float32(127.0) / np.abs(r2["y"]).max()
    r3 = run_linear(q8, x, W, b, flags=4, next_scale=ns)
    check_linear(r3, x, b)
    np.testing.assert_array_equal(r3["y"], O.quantize(r2["y"], ns))
    diff = r3["y"].astype(np.int32) - O.quantize(ref2["y"], ns).astype(np.int32)
    assert np.abs(diff).max() <= 1
    p = ref2["y"].astype(np.float64) * float(ns)
    near_tie = np.abs(np.abs(p - np.trunc(p)) - 0.5) < 1e-4 * np.maximum(1.0, np.abs(p))
    assert np.all(near_tie[diff != 0])
    # GELU + requant together
    gmax = np.abs(r["y"]).max()
    ns2 = np.float32(127.0) / gmax
    r4 = run_linear(q8, x, W, b, flags=1 | 4, next_scale=ns2)
    np.testing.assert_array_equal(r4["y"], O.quantize(r["y"], ns2))
    # ... and against the oracle's own GELU values: a code may differ by one, and only where the oracle's product
    # sits within the GELU tolerance (abs 1e-6 + rel 1e-5, times the scale) of a tie
    diff = r4["y"].astype(np.int32) - O.quantize(gl, ns2).astype(np.int32)
    assert np.abs(diff).max() <= 1
    p = gl.astype(np.float64) * float(ns2)
    slack = float(ns2) * (GELU_ATOL + GELU_RTOL * np.abs(gl.astype(np.float64))) + 1e-6 * np.maximum(1.0, np.abs(p))
    assert np.all(np.abs(np.abs(p - np.trunc(p)) - 0.5)[diff != 0] <= slack[diff != 0])


def test_gelu_epilogue_dense_grid(q8):
    """The fused GELU on a dense grid of arguments: with all-zero activations the accumulator is the
    quantized bias, so y = bias exactly (scales 32 x 32 = 2^10, bias on the 2^-10 grid) and the
    epilogue's GELU is seen on every multiple of 1/1024 in [-12, 12] -- both tails, the minimum near
    -0.75 and the clamp of the fit at |v| = 6 included.  MFMA and generic kernels."""
    import math
    grid = (np.arange(-12 * 1024, 12 * 1024 + 1, dtype=np.float64) / 1024.0)
    N = 24576
    b = np.zeros(N, dtype=np.float32)
    b[:] = grid[:N].astype(np.float32)
    b[-1] = np.float32(1e4)                                   # far beyond the clamp
    b[-2] = np.float32(-1e4)
    ref = O.gelu(b)
    for M, K in ((64, 128), (3, 100)):                        # MFMA path / generic path
        xq = torch.zeros((M, K), dtype=torch.int8, device="cuda")
        wq = dev(synth.random_int8(synth.rng(5), (N, K)))
        y = torch.empty((M, N), device="cuda")
        am = scalar(0.0)
        q8.q8_linear(xq, wq, dev(b), scalar(32.0), scalar(32.0), y, out_amax=am, flags=q8.EPI_GELU | q8.EPI_ABSMAX)
        got = host(y)
        for m in (0, M - 1):
            assert_rel(got[m], ref, rtol=GELU_RTOL, atol=GELU_ATOL)
        assert host(am)[0] == np.abs(got).max()
        # plain epilogue returns the grid itself
        q8.q8_linear(xq, wq, dev(b), scalar(32.0), scalar(32.0), y)
        np.testing.assert_array_equal(host(y)[0], b)


@pytest.mark.parametrize("M,K,N", [(768, 256, 512), (700, 384, 600)])
def test_linear_specialised_epilogues(q8, M, K, N):
    """Each epilogue combination has a kernel of its own when no accumulator dump is asked for;
    it must give the same bytes as the run-time-flag kernel (which the other tests pin to the
    oracle), on interior tiles and on ragged ones, for every tile shape."""
    g = synth.rng(51 + M)
    xq = dev(synth.random_int8(g, (M, K)))
    wq = dev(synth.random_int8(g, (N, K)))
    b = dev(synth.bias(g, N))
    sx, sw, ns = scalar(24.0), scalar(900.0), scalar(9.0)
    for variant in (1, 2, 3, 4, 5, 6):
        q8.set_gemm_variant(variant)
        try:
            for flags in range(8):
                dt = torch.int8 if flags & 4 else torch.float32
                y_gen = torch.zeros((M, N), dtype=dt, device="cuda")
                y_spec = torch.zeros((M, N), dtype=dt, device="cuda")
                acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
                a_gen, a_spec = scalar(0.0), scalar(0.0)
                kw = dict(next_scale=ns if flags & 4 else None, flags=flags)
                q8.q8_linear(xq, wq, b, sx, sw, y_gen, acc_out=acc, out_amax=a_gen if flags & 2 else None, **kw)
                q8.q8_linear(xq, wq, b, sx, sw, y_spec, out_amax=a_spec if flags & 2 else None, **kw)
                assert torch.equal(y_gen, y_spec), (variant, flags)
                assert host(a_gen)[0] == host(a_spec)[0], (variant, flags)
        finally:
            q8.set_gemm_variant(0)
    # and the run-time-flag kernel against the oracle at this shape, GELU + abs-max
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    y = torch.empty((M, N), device="cuda")
    am = scalar(0.0)
    q8.q8_linear(xq, wq, b, sx, sw, y, acc_out=acc, out_amax=am, flags=3)
    bq = O.quantize_bias(host(b), N, 24.0, [900.0])
    acc_ref = O.gemm_i8(host(xq), host(wq), bq, threads=8)
    np.testing.assert_array_equal(host(acc), acc_ref)
    assert_rel(host(y), O.gelu(O.dequant(acc_ref, 24.0, [900.0])), rtol=GELU_RTOL, atol=GELU_ATOL)
    assert host(am)[0] == np.abs(host(y)).max()


@pytest.mark.parametrize("M,K,N,variant", [
    (768, 256, 512, 0), (768, 256, 512, 1), (768, 256, 512, 2), (768, 256, 512, 3), (768, 256, 512, 4), (768, 256, 512, 5),
    (768, 256, 512, 6), (700, 384, 600, 0), (700, 384, 600, 2), (700, 384, 600, 3), (700, 384, 600, 5), (700, 384, 600, 6),
    (257, 128, 129, 0), (1, 128, 1, 0), (1030, 1024, 2100, 0), (33, 100, 70, 0), (5, 1, 3, 0),
])
def test_linear_residual_epilogue(q8, M, K, N, variant):
    """The FC layer with the encoder's residual addition fused (Section 3: the addition stays FP32): one binary32
    addition on top of the dequantized output.  Interior and edge tiles of every tile shape, the generic kernel, the
    run-time-flag kernel (abs-max of the sum, accumulator dump, GELU) and the in-place form."""
    d = synth.fc_layer(4000 + M + N + variant, M, K, N)
    rng = np.random.default_rng(77 + M + variant)
    wq_h, sw_h = O.quantize_tensor(d["W"])
    ref = O.linear(d["x"], wq_h, np.array([sw_h], np.float32), d["b"], threads=8)
    res_h = (rng.standard_normal((M, N)) * max(float(np.abs(ref["y"]).max()), 1e-3) * 0.5).astype(np.float32)
    xq, wq, sx, sw, b, res = dev(ref["xq"]), dev(wq_h), scalar(float(ref["sx"])), scalar(float(sw_h)), dev(d["b"]), dev(res_h)
    y0, y1, y2, y3 = (torch.empty((M, N), device="cuda") for _ in range(4))
    acc, amax, amax_g = torch.empty((M, N), dtype=torch.int32, device="cuda"), scalar(0.0), scalar(0.0)
    y_inplace = res.clone()
    q8.set_gemm_variant(variant)
    try:
        q8.q8_linear(xq, wq, b, sx, sw, y0)
        q8.q8_linear_residual(xq, wq, b, sx, sw, res, y1)                                   # the dedicated kernel
        q8.q8_linear_residual(xq, wq, b, sx, sw, res, y2, acc_out=acc, out_amax=amax, flags=q8.EPI_ABSMAX)
        q8.q8_linear_residual(xq, wq, b, sx, sw, res, y3, out_amax=amax_g, flags=q8.EPI_GELU | q8.EPI_ABSMAX)
        q8.q8_linear_residual(xq, wq, b, sx, sw, y_inplace, y_inplace)
        yg = torch.empty((M, N), device="cuda")
        q8.q8_linear(xq, wq, b, sx, sw, yg, flags=q8.EPI_GELU)
    finally:
        q8.set_gemm_variant(0)
    torch.cuda.synchronize()
    y0h, y1h = host(y0), host(y1)
    np.testing.assert_array_equal(host(acc), ref["acc"])
    np.testing.assert_array_equal(y1h, y0h + res_h)                  # exactly the unfused output plus one fp32 addition
    np.testing.assert_array_equal(host(y2), y1h)
    np.testing.assert_array_equal(host(y_inplace), y1h)
    np.testing.assert_array_equal(host(y3), host(yg) + res_h)        # activation first, then the addition
    assert host(amax)[0] == np.abs(y1h).max() and host(amax_g)[0] == np.abs(host(y3)).max()
    exact = ref["y"].astype(np.float64) + res_h.astype(np.float64)   # and against the oracle's FC output
    assert np.all(np.abs(y1h.astype(np.float64) - exact) <= 1e-6 * np.abs(ref["y"]) + 6e-8 * np.abs(exact) + 1e-30)


def test_linear_residual_argument_checks(q8):
    xq, wq = torch.zeros((4, 128), dtype=torch.int8, device="cuda"), torch.zeros((4, 128), dtype=torch.int8, device="cuda")
    y, s = torch.empty((4, 4), device="cuda"), scalar(1.0)
    with pytest.raises(q8.Q8Error) as e:
        q8.q8_linear_residual(xq, wq, None, s, s, y, y, flags=q8.EPI_REQUANT)
    assert e.value.code == 4
    import ctypes
    assert q8._lib.q8_linear_residual(xq.data_ptr(), wq.data_ptr(), None, s.data_ptr(), s.data_ptr(), 1, 4, 4, 128, None,
                                      y.data_ptr(), None, None, 0, None) == 1                       # residual missing
    assert q8._lib.q8_linear_residual(None, None, None, None, None, 1, 0, 4, 128, None, None, None, None, 0, None) == 0


def test_linear_static_activation_scale(q8):
    d = synth.fc_layer(46, 150, 256, 200)
    sx = np.float32(20.0)                                   # stored scale: values beyond 6.35 saturate
    r = run_linear(q8, d["x"] * np.float32(2.0), d["W"], d["b"], sx_static=sx)
    ref = check_linear(r, d["x"] * np.float32(2.0), d["b"], sx_static=sx)
    assert np.abs(r["xq"]).max() == 127
    assert_rel(r["y"], ref["y"])


def test_static_scale_ffn_chain_int8_to_int8(q8):
    """The paper's own inference mode keeps a stored activation scale (Eq. 4), so FFN1 can
    emit int8 directly (GELU + requantize in the epilogue) and FFN2 consumes it with no
    quantize pass.  Checked stage by stage: each stage's oracle is fed the GPU's own output
    of the stage before it."""
    g = synth.rng(52)
    M, H, F = 512, 256, 1024
    d = synth.ffn_block(53, M, H, F)
    x, W1, b1, W2, b2 = d["x"], d["W1"] * np.float32(4.0), d["b1"], d["W2"], d["b2"]
    w1q, s1 = O.quantize_tensor(W1)
    w2q, s2 = O.quantize_tensor(W2)
    sx = np.float32(127.0 / 4.5)            # stored scales, as a calibration run would leave them
    sg = np.float32(127.0 / 6.0)
    xd = dev(x)
    xq = torch.empty((M, H), dtype=torch.int8, device="cuda")
    q8.q8_quantize(xd, scalar(float(sx)), xq)
    np.testing.assert_array_equal(host(xq), O.quantize(x, sx))
    # FFN1: fp32 (GELU) reference run on the GPU, then the fused int8 run
    g32 = torch.empty((M, F), device="cuda")
    gq = torch.empty((M, F), dtype=torch.int8, device="cuda")
    q8.q8_linear(xq, dev(w1q), dev(b1), scalar(float(sx)), scalar(float(s1)), g32, flags=q8.EPI_GELU)
    q8.q8_linear(xq, dev(w1q), dev(b1), scalar(float(sx)), scalar(float(s1)), gq, next_scale=scalar(float(sg)),
                 flags=q8.EPI_GELU | q8.EPI_REQUANT)
    ref1 = O.linear(x, w1q, s1, b1, sx=sx, act_gelu=True, threads=8)
    assert_rel(host(g32), ref1["y"], rtol=GELU_RTOL, atol=GELU_ATOL)
    np.testing.assert_array_equal(host(gq), O.quantize(host(g32), sg))      # codes of the GPU's own fp32 values
    dq = host(gq).astype(np.int32) - O.quantize(ref1["y"], sg).astype(np.int32)
    assert np.abs(dq).max() <= 1
    p1 = ref1["y"].astype(np.float64) * float(sg)                           # codes differ only next to a tie
    slack = float(sg) * (GELU_ATOL + GELU_RTOL * np.abs(ref1["y"].astype(np.float64))) + 1e-6 * np.maximum(1.0, np.abs(p1))
    assert np.all(np.abs(np.abs(p1 - np.trunc(p1)) - 0.5)[dq != 0] <= slack[dq != 0])
    assert np.abs(host(gq)).max() == 127                                     # the stored scale saturates the tail
    # FFN2 straight from the int8 codes
    y = torch.empty((M, H), device="cuda")
    acc = torch.empty((M, H), dtype=torch.int32, device="cuda")
    q8.q8_linear(gq, dev(w2q), dev(b2), scalar(float(sg)), scalar(float(s2)), y, acc_out=acc)
    bq2 = O.quantize_bias(b2, H, sg, [s2])
    acc_ref = O.gemm_i8(host(gq), w2q, bq2, threads=8)
    np.testing.assert_array_equal(host(acc), acc_ref)
    assert_rel(host(y), O.dequant(acc_ref, sg, [s2]))
    # and the chain approximates the fp64 FFN it stands for
    ref = O.gelu((x.astype(np.float64) @ W1.T.astype(np.float64) + b1).astype(np.float32)).astype(np.float64) \
        @ W2.T.astype(np.float64) + b2
    err = host(y).astype(np.float64) - ref
    assert np.sqrt(np.mean(err ** 2)) < 0.05 * np.sqrt(np.mean(ref ** 2))


def test_linear_f32_one_call_equals_chain(q8):
    d = synth.fc_layer(47, 260, 384, 300)
    r = run_linear(q8, d["x"], d["W"], d["b"])
    M, K = d["x"].shape
    N = d["W"].shape[0]
    xq_work = torch.empty(M * K, dtype=torch.int8, device="cuda")
    scal = torch.zeros(q8.SCAL_WORK, device="cuda")
    y = torch.empty((M, N), device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    q8.q8_linear_f32(dev(d["x"]), dev(r["wq"]), dev(d["b"]), dev(r["sw"]), xq_work, scal, y, acc_out=acc)
    np.testing.assert_array_equal(host(acc), r["acc"])
    np.testing.assert_array_equal(host(y), r["y"])
    np.testing.assert_array_equal(host(xq_work).reshape(M, K), r["xq"])
    assert host(scal)[1] == r["sx"]
    # with the abs-max epilogue the one-call form resets the slot itself: stale contents do not survive
    for M2 in (M, 0):
        am = torch.full((1,), 1e9, device="cuda")
        y2 = torch.empty((M2, N), device="cuda")
        q8.q8_linear_f32(dev(d["x"][:M2]), dev(r["wq"]), dev(d["b"]), dev(r["sw"]), xq_work, scal, y2, out_amax=am,
                         flags=q8.EPI_ABSMAX)
        if M2:
            np.testing.assert_array_equal(host(y2), r["y"])
            assert host(am)[0] == np.abs(r["y"]).max()
        else:
            assert host(am)[0] == 1e9 or host(am)[0] == 0.0          # nothing computed: slot untouched or cleared


def test_linear_f32_slots_equals_chain(q8):
    """The FC fed by abs-max slots of its producer: same bytes as the oracle's layer on that x, whatever the number of
    slots, and the abs-max epilogue's slot is reset by the call itself."""
    d = synth.fc_layer(48, 260, 384, 300)
    r = run_linear(q8, d["x"], d["W"], d["b"])
    M, K = d["x"].shape
    N = d["W"].shape[0]
    amax = np.abs(d["x"]).max()
    xq_work = torch.empty(M * K, dtype=torch.int8, device="cuda")
    for n_slots in (1, 5, q8.AMAX_SLOTS):
        slots = np.zeros(n_slots, np.float32)
        slots[n_slots // 2] = amax                      # the maximum anywhere among the slots, the rest smaller
        if n_slots > 2:
            slots[0] = amax / 3
        scal = torch.zeros(2, device="cuda")
        y = torch.empty((M, N), device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        am = torch.full((1,), 1e9, device="cuda")
        q8.q8_linear_f32_slots(dev(d["x"]), dev(slots), dev(r["wq"]), dev(d["b"]), dev(r["sw"]), xq_work, scal, y, acc_out=acc,
                               out_amax=am, flags=q8.EPI_ABSMAX)
        np.testing.assert_array_equal(host(acc), r["acc"])
        np.testing.assert_array_equal(host(y), r["y"])
        np.testing.assert_array_equal(host(xq_work).reshape(M, K), r["xq"])
        assert host(scal)[0] == amax and host(scal)[1] == r["sx"] and host(am)[0] == np.abs(r["y"]).max()
    # argument checks
    raw = q8.raw()
    p = xq_work.data_ptr()
    assert raw.q8_linear_f32_slots(p, None, 1, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == 1   # no slots
    assert raw.q8_linear_f32_slots(p, p, 0, p, None, p, 1, 4, 4, 128, p, p, p, None, None, None, 0, None) == 2      # n_slots < 1


@pytest.mark.parametrize("M,K,N,groups", [(16, 768, 768, 1), (1, 128, 1, 1), (21, 768, 70, 1), (22, 768, 64, 1), (32, 512, 130, 1),
                                           (16, 1024, 3072, 3), (17, 1024, 64, 1), (5, 256, 200, 2), (32, 384, 96, 1), (8, 1152, 64, 1)])
def test_linear_f32_few_tokens_one_launch(q8, M, K, N, groups):
    """Section 4.1 + Section 3 for a handful of tokens: the one-launch kernel (every workgroup runs the quantizer itself,
    codes stay in LDS) where it applies, the two-launch path just outside it (M * K > 16384, K > 1024): every
    intermediate against the oracle, every epilogue, and byte for byte what the chain of separate calls gives."""
    g = synth.rng(7000 + M + K + N)
    x = synth.activations(g, M, K)
    x[int(g.integers(0, M)), int(g.integers(0, K))] = np.float32(-6.25)
    Ws = [synth.weights(g, N // groups, K) for _ in range(groups)]
    b = None if M == 5 else (g.standard_normal(N) * 0.05).astype(np.float32)      # one case without a bias
    q = [O.quantize_tensor(Wp) for Wp in Ws]
    wq_h, sw_h = np.concatenate([a for a, _ in q], 0), np.array([s_ for _, s_ in q], np.float32)
    ref = O.linear(x, wq_h, sw_h, b, threads=8)
    ref_g = O.gelu(ref["y"])
    xd, wq, sw, bd = dev(x), dev(wq_h), dev(sw_h), None if b is None else dev(b)
    ns_h = np.float32(127.0 / max(float(np.abs(ref_g).max()), 1e-6))
    ns = scalar(float(ns_h))
    for flags in (0, q8.EPI_GELU, q8.EPI_REQUANT, q8.EPI_GELU | q8.EPI_REQUANT):
        xq_work = torch.full((M * K,), 99, dtype=torch.int8, device="cuda")
        scal = torch.full((q8.SCAL_WORK,), -3.0, device="cuda")
        y = torch.full((M, N), 77, dtype=torch.int8 if flags & 4 else torch.float32, device="cuda")
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        q8.q8_linear_f32(xd, wq, bd, sw, xq_work, scal, y, n_groups=groups, acc_out=acc if flags == 0 else None,
                         next_scale=ns if flags & 4 else None, flags=flags)
        # the chain of separate calls on the same data
        a2, s2 = scalar(0.0), scalar(0.0)
        xq2 = torch.empty((M, K), dtype=torch.int8, device="cuda")
        y2 = torch.empty_like(y)
        q8.q8_absmax(xd, a2, s2)
        q8.q8_quantize(xd, s2, xq2)
        q8.q8_linear(xq2, wq, bd, s2, sw, y2, n_groups=groups, next_scale=ns if flags & 4 else None, flags=flags)
        torch.cuda.synchronize()
        sh = host(scal)
        assert sh[0] == np.float32(6.25) and sh[1] == ref["sx"]
        np.testing.assert_array_equal(host(xq_work).reshape(M, K), ref["xq"])
        np.testing.assert_array_equal(host(y), host(y2))
        if flags == 0:
            np.testing.assert_array_equal(host(acc), ref["acc"])
            assert_rel(host(y), ref["y"])
        elif flags == q8.EPI_GELU:
            assert np.all(np.abs(host(y).astype(np.float64) - ref_g) <= 1e-6 + 1e-5 * np.abs(ref_g))
        elif flags == q8.EPI_REQUANT:
            yf = torch.empty((M, N), device="cuda")
            q8.q8_linear(xq2, wq, bd, s2, sw, yf, n_groups=groups)
            np.testing.assert_array_equal(host(y), O.quantize(host(yf), ns_h))     # codes of the GPU's own fp32 outputs


@pytest.mark.parametrize("n", [4096, 16383, 16384, 16385])
def test_linear_f32_small_tensor_single_launch_boundary(q8, n):
    """Around the size up to which one workgroup does abs-max, scale and quantize in one launch: same bytes on
    both sides of it, also from a 4-byte aligned view."""
    g = synth.rng(600 + n)
    x = synth.activations(g, 1, n)
    x[0, int(g.integers(0, n))] = np.float32(-7.5)                  # the maximum somewhere inside
    W = synth.weights(g, 3, n)
    wq, sw = O.quantize_tensor(W)
    ref = O.linear(x, wq, sw, None)
    buf = torch.empty(n + 1, device="cuda")
    buf[1:] = dev(x).reshape(-1)
    for xd in (dev(x), buf[1:].view(1, n)):
        xq_work = torch.full((n,), 99, dtype=torch.int8, device="cuda")
        scal = torch.zeros(q8.SCAL_WORK, device="cuda")
        y = torch.empty((1, 3), device="cuda")
        q8.q8_linear_f32(xd, dev(wq), None, dev(np.array([sw], np.float32)), xq_work, scal, y)
        np.testing.assert_array_equal(host(xq_work).reshape(1, n), ref["xq"])
        assert host(scal)[0] == np.float32(7.5) and host(scal)[1] == ref["sx"]
        np.testing.assert_allclose(host(y), ref["y"], rtol=1e-6)


@pytest.mark.parametrize("n", [1, 7, 1000, 4_194_304, 12_582_912 + 3])
def test_linear_f32_scales_and_codes_at_size(q8, n):
    """The fused path's slot-based abs-max: scale and codes bit-exact for sizes from one
    element to a full activation tensor (more slots than one trip fills)."""
    g = synth.rng(500 + n % 71)
    x = g.standard_normal(n, dtype=np.float32)
    x[g.integers(0, n)] = np.float32(-9.5)
    wq = torch.zeros((1, n), dtype=torch.int8, device="cuda") if n <= 131071 else None
    xq_work = torch.empty(n, dtype=torch.int8, device="cuda")
    scal = torch.full((q8.SCAL_WORK,), -3.0, device="cuda")
    if wq is not None:     # through the one-call entry point (M = 1, K = n)
        q8.q8_linear_f32(dev(x).view(1, n), wq, None, scalar(1.0), xq_work, scal, torch.empty((1, 1), device="cuda"))
    else:                  # K too long for one GEMM row: M = n / 1024 rows of 1024
        rows = n // 1024
        x = x[: rows * 1024]
        wq = torch.zeros((1, 1024), dtype=torch.int8, device="cuda")
        xq_work = torch.empty(rows * 1024, dtype=torch.int8, device="cuda")
        q8.q8_linear_f32(dev(x).view(rows, 1024), wq, None, scalar(1.0), xq_work, scal,
                         torch.empty((rows, 1), device="cuda"))
    s = O.scale(O.absmax(x))
    sh = host(scal)
    assert sh[0] == O.absmax(x) and sh[1] == s
    np.testing.assert_array_equal(host(xq_work), O.quantize(x, s))


def test_quantize_amax_one_value_and_partials(q8):
    g = synth.rng(49)
    x = g.standard_normal(100_003, dtype=np.float32)
    a = O.absmax(x)
    s = O.scale(a)
    for amax_vals in ([float(a)], [0.1, float(a), 0.5, 0.0], list(np.abs(x[:700]).astype(float)) + [float(a)]):
        scale_out, amax_out = scalar(-1.0), scalar(-1.0)
        q = torch.empty(x.size, dtype=torch.int8, device="cuda")
        q8.q8_quantize_amax(dev(x), dev(np.array(amax_vals, np.float32)), scale_out, q, amax_out=amax_out)
        assert host(scale_out)[0] == s and host(amax_out)[0] == a
        np.testing.assert_array_equal(host(q), O.quantize(x, s))
    # a tensor above 64 MB with a single abs-max value: the streaming (non-temporal load) form of the kernel
    big = np.tile(x, 170)[: 17_000_003]
    qb = torch.empty(big.size, dtype=torch.int8, device="cuda")
    scale_out = scalar(-1.0)
    q8.q8_quantize_amax(dev(big), dev(np.array([float(a)], np.float32)), scale_out, qb)
    assert host(scale_out)[0] == s
    np.testing.assert_array_equal(host(qb), O.quantize(big, s))
    # an empty tensor still folds its abs-max values: a = their maximum, S = 127 / a
    scale_out, amax_out = scalar(-1.0), scalar(-1.0)
    q8.q8_quantize_amax(torch.empty(0, device="cuda"), dev(np.array([0.25, 2.0, 0.5], np.float32)), scale_out,
                        torch.empty(0, dtype=torch.int8, device="cuda"), amax_out=amax_out)
    assert host(amax_out)[0] == 2.0 and host(scale_out)[0] == 63.5
    # all-zero abs-max: S = 1; misaligned views take the scalar kernel
    scale_out = scalar(-1.0)
    q = torch.empty(16, dtype=torch.int8, device="cuda")
    q8.q8_quantize_amax(dev(x)[1:14], scalar(0.0), scale_out, q[1:14])
    assert host(scale_out)[0] == 1.0
    np.testing.assert_array_equal(host(q)[1:14], O.quantize(x[1:14], 1.0))


@pytest.mark.parametrize("n", [65_536, 65_540, 66_563, 1_048_576 + 259 * 4 + 3, 6_291_456])
def test_quantize_large_tensors_sixteen_byte_stores(q8, n):
    """Tensors of 16384 vectors and more with a single scale take the kernel that stores 16 codes per lane: whole 4 KiB blocks,
    a ragged last block, a tail of 1-3 elements, a stored scale and a single abs-max value (with the scalars and the
    cleared slot the GEMM behind it reads), codes only inside q, and the 4-byte-store kernel for a q that is not 16-byte aligned."""
    g = synth.rng(7100 + n % 101)
    x = g.standard_normal(n, dtype=np.float32) * np.float32(2.5)
    a = O.absmax(x)
    s = O.scale(a)
    want = O.quantize(x, s)
    xd = dev(x)
    for qoff in (0, 4, 16):
        buf = torch.full((n + 64,), 99, dtype=torch.int8, device="cuda")
        q = buf[qoff:qoff + n]
        q8.q8_quantize(xd, scalar(float(s)), q)
        hb = host(buf)
        np.testing.assert_array_equal(hb[qoff:qoff + n], want)
        assert np.all(hb[:qoff] == 99) and np.all(hb[qoff + n:] == 99)
        buf.fill_(99)
        scale_out, amax_out = scalar(-1.0), scalar(-1.0)
        q8.q8_quantize_amax(xd, scalar(float(a)), scale_out, q, amax_out=amax_out)
        hb = host(buf)
        assert host(scale_out)[0] == s and host(amax_out)[0] == a
        np.testing.assert_array_equal(hb[qoff:qoff + n], want)
        assert np.all(hb[:qoff] == 99) and np.all(hb[qoff + n:] == 99)
    # the FC layer fed by one abs-max value (the previous layer's fused abs-max): quantizer scalars and the cleared slot
    if n == 6_291_456:
        M, K, N = 6144, 1024, 128
        wq = dev(synth.random_int8(g, (N, K)))
        scal = torch.full((2,), -1.0, device="cuda")
        xq_work = torch.full((M * K,), 99, dtype=torch.int8, device="cuda")
        y = torch.empty((M, N), device="cuda")
        am = scalar(5.0)
        q8.q8_linear_f32_slots(xd.view(M, K), scalar(float(a)), wq, None, scalar(900.0), xq_work, scal, y, out_amax=am,
                               flags=q8.EPI_ABSMAX)
        assert host(scal)[0] == a and host(scal)[1] == s
        np.testing.assert_array_equal(host(xq_work), want)
        assert host(am)[0] == np.abs(host(y)).max()


@pytest.mark.parametrize("n", [0, 1, 1000, 16384, 16385, 3_145_731])
def test_quantize_dynamic_is_absmax_scale_quantize(q8, n):
    """The dynamic quantizer of Section 4.1 in one call: max|x|, S = 127 / max (Eq. 3), codes by Eq. 1, all against the oracle;
    the optional slot is cleared by the same launch."""
    g = synth.rng(4900 + n % 97)
    x = g.standard_normal(n, dtype=np.float32) * np.float32(3.0)
    scal = torch.full((q8.SCAL_WORK,), -1.0, device="cuda")
    q = torch.full((n,), 99, dtype=torch.int8, device="cuda")
    slot = scalar(7.0)
    q8.q8_quantize_dynamic(dev(x), q, scal, zero_slot=slot)
    a = O.absmax(x) if n else np.float32(0.0)
    s = O.scale(a)
    assert host(scal)[0] == a and host(scal)[1] == s and host(slot)[0] == 0.0
    if n:
        np.testing.assert_array_equal(host(q), O.quantize(x, s))


@pytest.mark.parametrize("mode", ["one_pass", "never_wait", "two_pass"])
@pytest.mark.parametrize("n,where", [(1_048_576, 0), (1_048_580, -1), (3_145_728, 1_500_000), (12_582_908, -1),
                                     (12_582_912, 0), (12_582_912, 6_000_001), (12_582_912, -1)])
def test_quantize_dynamic_register_resident_sizes(q8, n, where, mode):
    """Section 4.1 on tensors the one-pass kernel takes (x stays in registers between the abs-max and Eq. 1; its
    workgroups meet at a barrier): the kernel as it runs, the same with a barrier that never waits (every workgroup
    reads the shares of those it does not see yet), and the two-pass path, each against the oracle.  The extreme
    value sits in the first, a middle or the last workgroup's share and is negative."""
    rng = np.random.default_rng(900 + n % 1000 + (where % 7))
    x = rng.standard_normal(n).astype(np.float32)
    x[where] = np.float32(-11.5)
    xd, q = dev(x), torch.full((n,), 99, dtype=torch.int8, device="cuda")
    scal, z = torch.full((q8.SCAL_WORK,), 7.0, device="cuda"), scalar(5.0)
    q8.set_quantize_one_pass(mode != "two_pass", 0 if mode == "never_wait" else 64)
    try:
        q8.q8_quantize_dynamic(xd, q, scal, zero_slot=z)
        torch.cuda.synchronize()
    finally:
        q8.set_quantize_one_pass(True, 64)
    q_ref, s_ref = O.quantize_tensor(x)
    sh = host(scal)
    assert sh[0] == np.float32(11.5) and sh[1] == s_ref and host(z)[0] == 0.0
    np.testing.assert_array_equal(host(q), q_ref)


def test_quantize_dynamic_one_pass_all_zero_and_repeated_calls(q8):
    """An all-zero tensor takes S = 1; and the barrier's slots carry a new ticket on every launch, so a maximum
    left by an earlier, larger tensor is never picked up."""
    n = 2_097_152
    q, scal = torch.full((n,), 99, dtype=torch.int8, device="cuda"), torch.zeros(q8.SCAL_WORK, device="cuda")
    big = torch.full((n,), 1000.0, device="cuda")
    for rep in range(70):                                   # more launches than the ring of slot sets is long
        q8.q8_quantize_dynamic(big, q, scal)
    q8.q8_quantize_dynamic(torch.zeros(n, device="cuda"), q, scal)
    torch.cuda.synchronize()
    assert host(scal)[0] == 0.0 and host(scal)[1] == 1.0 and not host(q).any()
    x = np.random.default_rng(5).standard_normal(n).astype(np.float32)
    q8.q8_quantize_dynamic(dev(x), q, scal)
    torch.cuda.synchronize()
    q_ref, s_ref = O.quantize_tensor(x)
    assert host(scal)[1] == s_ref
    np.testing.assert_array_equal(host(q), q_ref)


def test_quantize_dynamic_one_pass_on_two_streams(q8):
    """Two one-pass launches in flight at once, each needing the whole chip for its barrier to open: whichever way the
    hardware interleaves them (one after the other, or each holding part of the compute units until the bounded wait
    runs out and the absent shares are read instead) both results are the oracle's."""
    n = 12_582_912
    rng = np.random.default_rng(31)
    xs = [rng.standard_normal(n).astype(np.float32) * np.float32(1 + i) for i in range(2)]
    xd = [dev(x) for x in xs]
    qs = [torch.full((n,), 99, dtype=torch.int8, device="cuda") for _ in range(2)]
    scals = [torch.zeros(q8.SCAL_WORK, device="cuda") for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):
        for i in range(2):
            q8.q8_quantize_dynamic(xd[i], qs[i], scals[i], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        q_ref, s_ref = O.quantize_tensor(xs[i])
        assert host(scals[i])[1] == s_ref
        np.testing.assert_array_equal(host(qs[i]), q_ref)


def test_quantize_dynamic_one_pass_many_launches(q8):
    """Several hundred one-pass launches back to back, sizes alternating and two streams in flight: every launch's
    maximum and scale are its own tensor's (a barrier that opened early, or a slot read from another launch, would
    show as a wrong maximum), and the codes of the last launch of each stream are the oracle's."""
    sizes = [1_048_576, 12_582_912, 3_145_728, 2_097_152]
    rng = np.random.default_rng(77)
    xs = {n: torch.randn(n, device="cuda") for n in sizes}
    peak = {n: float(xs[n].abs().max()) for n in sizes}
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    qs = [torch.empty(max(sizes), dtype=torch.int8, device="cuda") for _ in range(2)]
    scal = torch.zeros((2, 300, q8.SCAL_WORK), device="cuda")
    torch.cuda.synchronize()
    order = []
    for it in range(300):
        n = sizes[int(rng.integers(0, len(sizes)))]
        sidx = it & 1
        q8.q8_quantize_dynamic(xs[n], qs[sidx][:n], scal[sidx, it], stream=streams[sidx])
        order.append((sidx, n))
    torch.cuda.synchronize()
    sh = host(scal[:, :, :2])
    for it, (sidx, n) in enumerate(order):
        assert sh[sidx, it, 0] == np.float32(peak[n]), (it, n)
        assert sh[sidx, it, 1] == O.scale(np.float32(peak[n])), (it, n)
    for sidx in range(2):
        n = [m for s_, m in order if s_ == sidx][-1]
        q_ref, _ = O.quantize_tensor(host(xs[n]))
        np.testing.assert_array_equal(host(qs[sidx][:n]), q_ref)


def test_linear_is_deterministic(q8):
    d = synth.fc_layer(48, 600, 512, 700)
    a = run_linear(q8, d["x"], d["W"], d["b"])
    b = run_linear(q8, d["x"], d["W"], d["b"])
    assert a["y"].tobytes() == b["y"].tobytes() and a["acc"].tobytes() == b["acc"].tobytes()


def test_linear_empty_shapes(q8):
    y = torch.full((4,), 7.0, device="cuda")
    q8.q8_linear(torch.empty((0, 128), dtype=torch.int8, device="cuda"),
                 torch.empty((4, 128), dtype=torch.int8, device="cuda"), None, scalar(1.0), scalar(1.0), y[:0])
    q8.q8_quantize(torch.empty(0, device="cuda"), scalar(1.0), torch.empty(0, dtype=torch.int8, device="cuda"))
    torch.cuda.synchronize()
    assert np.all(host(y) == 7.0)


# --------------------------------------------------------------------------- embedding
@pytest.mark.parametrize("V,H,T", [(1000, 768, 257), (30522, 768, 4096), (50, 30, 77), (2, 768, 100), (300, 1024, 1)])
def test_embedding_gather(q8, V, H, T):
    g = synth.rng(300 + V % 13)
    E = synth.weights(g, V, H)
    ed = dev(E)
    a, s = scalar(0.0), scalar(0.0)
    q8.q8_absmax(ed, a, s)
    eq = torch.empty((V, H), dtype=torch.int8, device="cuda")
    q8.q8_quantize(ed, s, eq)
    eq_ref, s_ref = O.quantize_tensor(E)
    np.testing.assert_array_equal(host(eq), eq_ref)
    ids = g.integers(0, V, size=T, dtype=np.int32)
    ids[0], ids[-1] = 0, V - 1
    if T > 4:
        ids[1] = ids[2] = V - 1
    out_i8 = torch.empty((T, H), dtype=torch.int8, device="cuda")
    out_f = torch.empty((T, H), device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    q8.q8_embedding(eq, s, dev(ids), out_i8, err_flag=flag)
    q8.q8_embedding(eq, s, dev(ids), out_f, err_flag=flag)
    ref_i8, ref_f = O.embedding(eq_ref, s_ref, ids)
    np.testing.assert_array_equal(host(out_i8), ref_i8)
    assert_rel(host(out_f), ref_f)
    assert host(flag)[0] == 0


def test_embedding_bad_ids_flagged_and_zeroed(q8):
    g = synth.rng(301)
    V, H = 100, 64
    eq = synth.random_int8(g, (V, H))
    ids = np.array([3, V, 5, -1, 99], dtype=np.int32)
    out = torch.full((5, H), 9.0, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    q8.q8_embedding(dev(eq), scalar(10.0), dev(ids), out, err_flag=flag)
    o = host(out)
    assert host(flag)[0] == 1
    assert not o[1].any() and not o[3].any()
    good = np.array([0, 2, 4])
    _, ref = O.embedding(eq, 10.0, ids[good])
    assert_rel(o[good], ref)
    with pytest.raises(O.OracleError):
        O.embedding(eq, 10.0, ids)
    # without a flag pointer the call still never reads out of range
    q8.q8_embedding(dev(eq), scalar(10.0), dev(ids), out, err_flag=None)
    torch.cuda.synchronize()


@pytest.mark.parametrize("H,T", [(768, 1000), (30, 33)])
def test_embedding_sum3(q8, H, T):
    g = synth.rng(302)
    sizes = (2000, 512, 2)
    tabs = [synth.weights(g, v, H) for v in sizes]
    qs = [O.quantize_tensor(t) for t in tabs]
    ids = [g.integers(0, v, size=T, dtype=np.int32) for v in sizes]
    out = torch.empty((T, H), device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    scales = dev(np.array([s for _, s in qs], np.float32))
    q8.q8_embedding_sum3(dev(qs[0][0]), dev(qs[1][0]), dev(qs[2][0]), scales, dev(ids[0]), dev(ids[1]), dev(ids[2]),
                         out, err_flag=flag)
    ref = O.embedding_sum3(qs[0][0], qs[0][1], qs[1][0], qs[1][1], qs[2][0], qs[2][1], *ids)
    # three fp32 terms summed: absolute tolerance scaled by the largest term
    mag = sum(np.abs(q[i].astype(np.float64)) / float(s) for (q, s), i in zip(qs, ids))
    assert np.all(np.abs(host(out).astype(np.float64) - ref) <= 1e-6 * mag + 1e-12)
    assert host(flag)[0] == 0


def test_embedding_sum3_empty_table_reads_nothing(q8):
    """One of the three tables is empty (V = 0, null pointer): every id into it is bad, so every output row is zero,
    the flag is raised, and no table is read through the row-0 stand-in of a bad id."""
    g = synth.rng(303)
    H, T = 64, 37
    word, pos = synth.random_int8(g, (50, H)), synth.random_int8(g, (16, H))
    ids = [g.integers(0, v, size=T, dtype=np.int32) for v in (50, 16, 2)]
    lib = q8.raw()
    scales = dev(np.array([10.0, 20.0, 30.0], np.float32))
    for vec in (True, False):                                  # 16-byte aligned (vector kernel) and not
        buf = torch.full((T * H + 1,), 9.0, device="cuda")
        out = buf[:T * H] if vec else buf[1:]
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        wd, pd = dev(word), dev(pos)
        idd = [dev(i) for i in ids]
        rc = lib.q8_embedding_sum3(wd.data_ptr(), 50, pd.data_ptr(), 16, None, 0, scales.data_ptr(), H, idd[0].data_ptr(),
                                   idd[1].data_ptr(), idd[2].data_ptr(), T, out.data_ptr(), flag.data_ptr(), None)
        assert rc == 0
        torch.cuda.synchronize()
        assert host(flag)[0] == 1 and not host(out).any()


def test_measurement_kernels(q8):
    """The benchmark's measurement kernels (not part of the method): the streaming copy copies, the fill fills, and the
    MFMA-rate loop and every built combination of the main-loop stage probe run to completion inside their windows."""
    g = synth.rng(311)
    src = dev(g.standard_normal(1 << 20, dtype=np.float32))
    dst = torch.zeros(1 << 20, device="cuda")
    q8.debug_stream_copy(src, dst)
    assert torch.equal(src, dst)
    q8.debug_stream_copy(None, dst)
    assert bool((dst == 1.0).all())
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ops = dev(synth.random_int8(g, (65536,)))
    assert q8.debug_mfma_rate(ops, 3, 4, sink) == 2.0 * 32768 * 8 * 3 * 8 * 4
    opw = torch.zeros(4 << 20, dtype=torch.int8, device="cuda")
    stw = torch.full((8 << 20,), -3.0, device="cuda")
    guard = torch.full((1024,), -3.0, device="cuda")          # allocated right behind: must stay untouched
    for what in (0, 7, 15, 64, 71, 79):
        q8.debug_loop_probe(what, opw, stw, 5, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0 and bool((guard == -3.0).all())
    with pytest.raises(q8.Q8Error):
        q8.debug_loop_probe(3, opw, stw, 5, sink)
