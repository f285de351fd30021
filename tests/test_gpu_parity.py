"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Bars: dequantized weights bit-exact; outputs within max relative error 2e-3 (see gpu_util)."""
import numpy as np
import pytest

from oracle import rwkvq_oracle as orc
from paper_2505_03803_amd import binding as B
from paper_2505_03803_amd import synth

import gpu_util as G

pytestmark = pytest.mark.gpu


def make(fmt, N, K, seed):
    rng = np.random.default_rng(seed)
    if fmt == "sq":
        return synth.gen_sq(rng, N, K)
    return synth.gen_vq(rng, N, K, 6 if fmt == "vq6" else 8)


def acts(M, K, dtype, seed):
    return synth.gen_activations(np.random.default_rng(seed + 99), M, K, dtype)


FORCE = {None: B.SMALL_BATCH_AUTO, "stream": B.SMALL_BATCH_STREAM, "mfma": B.SMALL_BATCH_MATRIX_CORES}



@pytest.fixture(params=["columns-split", "columns-split, table of first workgroups", "256-row-workgroups", "128-row-workgroups"])
def stretches(request, options):
    """Batch 2..32 on the streaming kernels has three forms, chosen by the size of the launch: one workgroup per 32
    rows whose wavefronts split the columns and fetch their activation fragments themselves (small launches, batch
    <= 16: RWKVQ_OPT_STREAM_SPLIT_MAX_WORK), workgroups of 128 rows that share a staged activation tile, and
    workgroups of two such stretches (large launches: RWKVQ_OPT_STREAM_TWO_PASS_MIN_WGS).  The test shapes are small
    launches, so each form is forced in turn.  The column-split form finds matrix and stretch in a two-dimensional grid
    when the launch holds at most eight matrices, and in the table of first workgroups otherwise: both are forced."""
    form = request.param
    options(B.OPT_STREAM_SPLIT_MAX_WORK, 1000000 if form.startswith("columns-split") else 1)
    options(B.OPT_SPLIT_GRID_2D, 2 if form.endswith("table of first workgroups") else 1)
    options(B.OPT_STREAM_TWO_PASS_MIN_WGS, 1 if form == "256-row-workgroups" else 1000000)
    return form


SMALL = [("sq", 48, 768), ("sq", 256, 256), ("vq6", 256, 768), ("vq6", 512, 256), ("vq8", 256, 768),
         ("vq8", 512, 512)]


# ------------------------------------------------------------------ dequantization

@pytest.mark.parametrize("fmt,N,K", SMALL)
@pytest.mark.parametrize("native", [False, True])
def test_dequant_bit_exact(fmt, N, K, native):
    print(f"dequant {fmt} N={N} K={K} native={native}", flush=True)
    mat = make(fmt, N, K, 1)
    want = orc.dequant(mat)
    dm = B.upload(mat, native=native)
    got = G.gpu_dequant(dm)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    for name, code in (("bf16", B.BF16), ("f16", B.F16)):
        got16 = G.gpu_dequant(dm, code)
        want16 = orc.round_weights(want, name)
        back = orc.widen(got16, name)
        assert np.array_equal(back.view(np.uint32), want16.view(np.uint32)), name


def test_dequant_rounding_order_cases(golden_dir):
    # tiny zero points, where (q - z) itself rounds: the kernel must subtract, then multiply
    import os
    rows = [l.split() for l in open(os.path.join(golden_dir, "sq_rounding_cases.txt")) if not l.startswith("#")]
    mat = make("sq", 16, 256, 3)
    mat.codes[:] = 0
    expect = {}
    for i, (tag, q, zb, sb, a, *_rest) in enumerate(rows):
        n = i
        mat.scales[n, :] = int(sb, 16)
        mat.zeros[n, :] = int(zb, 16)
        mat.codes[n, 0] = int(q)            # code of column 0 = low 3 bits of word 0
        expect[n] = int(a, 16)
    for native in (False, True):
        got = G.gpu_dequant(B.upload(mat, native=native)).view(np.uint32)
        for n, a in expect.items():
            assert int(got[n, 0]) == a
    assert np.array_equal(orc.dequant(mat).view(np.uint32), got)


# ------------------------------------------------------------------ GEMV / GEMM on small shapes

@pytest.mark.parametrize("fmt,N,K", SMALL)
@pytest.mark.parametrize("M", [1, 3, 4, 7, 16])
@pytest.mark.parametrize("xdt", ["f16", "bf16"])
def test_decode_small(fmt, N, K, M, xdt, stretches):
    print(f"decode {fmt} N={N} K={K} M={M} x={xdt} two-pass threshold {stretches}", flush=True)
    mat = make(fmt, N, K, 2)
    x = acts(M, K, xdt, M)
    y = G.gpu_gemm(B.upload(mat, native=True), x, xdt)
    G.check_outputs(y, mat, x, xdt, fed=None, tight=2e-5)


@pytest.mark.parametrize("fmt,N,K", [("sq", 176, 512), ("sq", 272, 768), ("sq", 400, 256), ("vq6", 768, 512), ("vq8", 768, 768)])
@pytest.mark.parametrize("M", [2, 16, 17, 24, 32])
@pytest.mark.parametrize("xdt", ["f16", "bf16"])
def test_decode_batched_row_stretches(fmt, N, K, M, xdt, options, stretches):
    """Batch 2..32: a workgroup covers 256 rows of W as two stretches of 128 that share each staged activation
    tile.  Row counts that end inside the first stretch, inside the second, and one row tile into the next
    workgroup (SQ rows come in sixteens; VQ in blocks of 256, here three blocks).  M = 17 and 24 leave the second
    group of sixteen batch rows of the 32-row instances partly filled.  The streaming kernels are
    forced (left alone the dispatcher may send M > 16 to the matrix cores, which round the weights)."""
    print(f"decode row stretches {fmt} N={N} K={K} M={M} x={xdt} two-pass threshold {stretches}", flush=True)
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_STREAM)
    mat = make(fmt, N, K, 12)
    x = acts(M, K, xdt, N + M)
    y = G.gpu_gemm(B.upload(mat, native=True), x, xdt)
    G.check_outputs(y, mat, x, xdt, fed=None, tight=2e-5)


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
@pytest.mark.parametrize("N,K", [(256, 256), (256, 3584), (4096, 512), (4096, 1792), (8192, 256), (8192, 1280), (16384, 512), (65536, 256)])
@pytest.mark.parametrize("grid", ["matrix-by-row-tile grid", "table of first workgroups"])
def test_decode_batch1_launch_shapes(fmt, N, K, grid, options):
    """Batch 1 picks its kernel by the number of 16-row tiles in the launch: 16, 8 or 4 wavefronts
    per tile with the column tiles dealt round-robin (small launches), or one wavefront per tile
    (2048 tiles and more).  Rows with fewer column tiles than wavefronts, and
    tile counts that do not divide, are part of the sweep.  A small launch of few matrices finds its matrix
    and row tile in a two-dimensional grid; the table that launches of more than eight matrices use is forced too."""
    print(f"decode shapes {fmt} N={N} K={K} {grid}", flush=True)
    options(B.OPT_SPLIT_GRID_2D, 1 if grid.startswith("matrix") else 2)
    mat = make(fmt, N, K, 8)
    x = acts(1, K, "f16", N + K)
    y = G.gpu_gemm(B.upload(mat, native=True), x, "f16")
    G.check_outputs(y, mat, x, "f16", fed=None, tight=2e-5)


@pytest.mark.parametrize("fmt,N,K", [("sq", 256, 768), ("vq6", 256, 768), ("vq8", 512, 512)])
@pytest.mark.parametrize("M", [17, 256, 300])
@pytest.mark.parametrize("xdt", ["bf16", "f16"])
def test_prefill_small(fmt, N, K, M, xdt, options):
    print(f"prefill {fmt} N={N} K={K} M={M} x={xdt}", flush=True)
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_MATRIX_CORES)     # M = 17 on the matrix cores, whatever the estimate says
    mat = make(fmt, N, K, 4)
    x = acts(M, K, xdt, M)
    y = G.gpu_gemm(B.upload(mat, native=True), x, xdt)
    G.check_outputs(y, mat, x, xdt, fed=xdt, tight=2e-5)


@pytest.mark.parametrize("fmt,N,K", SMALL)
@pytest.mark.parametrize("M", [1, 9])
def test_reference_kernel_canonical(fmt, N, K, M):
    print(f"ref {fmt} N={N} K={K} M={M}", flush=True)
    mat = make(fmt, N, K, 5)
    x = acts(M, K, "f16", M)
    y = G.gpu_gemm(B.upload(mat, native=False), x, "f16")
    G.check_outputs(y, mat, x, "f16", fed=None, tight=2e-5)


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
def test_one_hot_returns_weight_column(fmt):
    """Batch 1 with a one-hot activation vector returns one column of Deq(W), bit for bit (every
    product but one is an exact zero), for every column of two tiles: each column goes through its
    own unpack position and its own lane of the activation broadcast."""
    mat = make(fmt, 256, 512, 6)
    w = orc.dequant(mat)
    dm = B.upload(mat, native=True)
    for k in range(512):
        x = np.zeros((1, 512), np.float32)
        x[0, k] = 1.0
        y = G.gpu_gemm(dm, synth.f32_to_f16_bits(x), "f16")[0]
        assert np.array_equal(y, w[:, k].astype(np.float64)), f"column {k}"


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
def test_one_hot_batch4(fmt):
    """The same through the matrix-core path (batch 4): row m selects column 37 m + 3.  The SQ
    codes enter the MFMA as 8 + q, so (8 + q) - (z + 8) can round once more than q - z."""
    mat = make(fmt, 256, 512, 6)
    w = orc.dequant(mat)
    dm = B.upload(mat, native=True)
    x = np.zeros((4, 512), np.float32)
    cols = [37 * m + 3 for m in range(4)]
    for m, k in enumerate(cols):
        x[m, k] = 1.0
    y = G.gpu_gemm(dm, synth.f32_to_f16_bits(x), "f16")
    for m, k in enumerate(cols):
        if fmt == "sq":
            assert np.allclose(y[m], w[:, k], rtol=1e-6, atol=0)
        else:
            assert np.array_equal(y[m], w[:, k].astype(np.float64))


@pytest.mark.parametrize("ydt", ["f16", "bf16"])
def test_output_rounding(ydt):
    mat = make("sq", 256, 512, 7)
    x = acts(2, 512, "f16", 1)
    dm = B.upload(mat, native=True)
    y32 = G.gpu_gemm(dm, x, "f16", B.F32)
    y16 = G.gpu_gemm(dm, x, "f16", B.DTYPES[ydt])
    want = orc.narrow(y32.astype(np.float32), ydt)
    assert np.array_equal(y16, want)


def test_dispatch_equals_single_calls():
    torch = G.torch_()
    mats = [make("sq", 256, 768, 10), make("vq6", 512, 256, 11), make("vq8", 256, 512, 12),
            make("sq", 48, 256, 13), make("vq6", 256, 1024, 14)]
    for M, xdt in ((1, "f16"), (4, "bf16"), (16, "bf16"), (40, "bf16")):
        dms = [B.upload(m, native=True) for m in mats]
        xs = [G.to_dev_bits(acts(M, m.K, xdt, i)) for i, m in enumerate(mats)]
        ys = [torch.empty((M, m.N), dtype=torch.float32, device="cuda") for m in mats]
        table = B.DispatchTable([d.desc() for d in dms], xs, ys)
        B.rwkvq_linear_dispatch(table, M, B.DTYPES[xdt], B.F32)
        torch.cuda.synchronize()
        for dm, x, y in zip(dms, xs, ys):
            single = B.gemm(dm, x, M, B.DTYPES[xdt], B.F32)
            torch.cuda.synchronize()
            if M == 1:      # the batch-1 kernel is picked by launch size: same sums, possibly another order
                assert (single - y).abs().max() <= 4e-6 * y.abs().max()
            else:
                assert torch.equal(single, y)


@pytest.mark.parametrize("M", [1, 4, 40])
def test_dispatch_many_matrices(M):
    """300 small matrices in one table: the decode launch holds 256 descriptors (four passes of the
    workgroup -> matrix look-up) and splits after them; the prefill launches split at 64 per format.
    Every output must equal the single-matrix call's (bit for bit on the matrix-core paths)."""
    torch = G.torch_()
    kinds = ("sq", "vq6", "vq8")
    shapes = ((48, 256), (256, 256), (256, 512), (32, 256), (512, 256))
    base = [make(kinds[i % 3], *(shapes[i % 5] if kinds[i % 3] == "sq" else (256, 256 + 256 * (i % 2))), 100 + i)
            for i in range(15)]
    dbase = [B.upload(m, native=True) for m in base]
    n = 300
    xs = [G.to_dev_bits(acts(M, base[i % 15].K, "f16", 200 + i)) for i in range(n)]
    ys = [torch.empty((M, base[i % 15].N), dtype=torch.float32, device="cuda") for i in range(n)]
    table = B.DispatchTable([dbase[i % 15].desc() for i in range(n)], xs, ys)
    B.rwkvq_linear_dispatch(table, M, B.F16, B.F32)
    torch.cuda.synchronize()
    def same(a, b):
        # batch 1 picks its kernel by launch size (a single call splits the columns over several
        # wavefronts, the big launch does not): the binary32 sums differ in their order only
        if M == 1:
            return bool((a - b).abs().max() <= 4e-6 * b.abs().max())
        return torch.equal(a, b)
    for i in list(range(0, n, 7)) + [n - 1]:
        single = B.gemm(dbase[i % 15], xs[i], M, B.F16, B.F32)
        torch.cuda.synchronize()
        assert same(single, ys[i]), i


# ------------------------------------------------------------------ the configurations

def test_config1_full():
    mat, x = synth.config1()
    dm = B.upload(mat, native=True)
    assert np.array_equal(G.gpu_dequant(dm).view(np.uint32), orc.dequant(mat).view(np.uint32))
    y = G.gpu_gemm(dm, x, "f16")
    print("config1", G.check_outputs(y, mat, x, "f16", tight=2e-5), flush=True)


def test_config2_full():
    mat, x = synth.config2()
    dm = B.upload(mat, native=True)
    assert np.array_equal(G.gpu_dequant(dm).view(np.uint32), orc.dequant(mat).view(np.uint32))
    y = G.gpu_gemm(dm, x, "f16")
    print("config2", G.check_outputs(y, mat, x, "f16", tight=2e-5), flush=True)


def _stack_layer_check(config, M, n_layers, rows=None, fed=None, tight=None):
    """Run the first layers of a stack through one rwkvq_linear_dispatch call and check every
    matrix; with `rows`, only those activation rows are checked against the oracle."""
    torch = G.torch_()
    xdt = synth.STACKS[config][4]
    items = list(synth.stack(config, M, n_layers=n_layers))
    dms = [B.upload(m, native=True) for m, _ in items]
    xs = [G.to_dev_bits(x) for _, x in items]
    ys = [torch.empty((M, m.N), dtype=torch.float32, device="cuda") for m, _ in items]
    table = B.DispatchTable([d.desc() for d in dms], xs, ys)
    B.rwkvq_linear_dispatch(table, M, B.DTYPES[xdt], B.F32)
    torch.cuda.synchronize()
    worst = (0.0, 0.0)
    for (mat, x), dm, y in zip(items, dms, ys):
        got = G.gpu_dequant(dm)
        assert np.array_equal(got.view(np.uint32), orc.dequant(mat).view(np.uint32)), mat.name
        del got
        yy = y.cpu().numpy().astype(np.float64)
        if rows is not None:
            yy, x = yy[rows], x[rows]
        g = G.check_outputs(yy, mat, x, xdt, fed=fed, tight=tight)
        worst = (max(worst[0], g[0]), max(worst[1], g[1]))
        print(f"  cfg{config} M={M} {mat.name} {mat.kind}{mat.kbits or ''} g1={g[0]:.2e} g2={g[1]:.2e}", flush=True)
    return worst


def test_config3_decode_layers():
    print("config3", _stack_layer_check(3, 1, n_layers=2, tight=2e-5), flush=True)


def test_config4_prefill_layer_sampled_rows():
    rows = np.random.default_rng(0).choice(2048, size=8, replace=False)
    print("config4", _stack_layer_check(4, 2048, n_layers=1, rows=np.sort(rows), fed="bf16", tight=2e-5), flush=True)


@pytest.mark.parametrize("M", [1, 16])
def test_config5_decode_layer(M):
    print("config5", M, _stack_layer_check(5, M, n_layers=1, tight=2e-5), flush=True)


def test_config5_prefill_layer_sampled_rows():
    rows = np.sort(np.random.default_rng(1).choice(4096, size=4, replace=False))
    print("config5 prefill", _stack_layer_check(5, 4096, n_layers=1, rows=rows, fed="bf16", tight=2e-5), flush=True)


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
@pytest.mark.parametrize("xdt", ["bf16", "f16"])
@pytest.mark.parametrize("N,K,M", [(256, 512, 64), (512, 768, 200), (256, 1024, 256), (512, 512, 300), (768, 256, 129)])
def test_prefill_both_tile_heights(fmt, xdt, N, K, M, options):
    """The matrix-core kernel exists with 256 and with 128 rows of x per workgroup (the launcher picks
    by how many tiles a launch has); both are forced in turn through rwkvq_set_option.  Same order of summation over k: the same bits, and each against the oracle."""
    torch = G.torch_()
    mat = make(fmt, N, K, 7)
    x = acts(M, K, xdt, M + 1)
    dm = B.upload(mat, native=True)
    ys = {}
    for bm in ("128", "256"):
        print(f"prefill tile height {bm}: {fmt} N={N} K={K} M={M} x={xdt}", flush=True)
        options(B.OPT_PREFILL_TILE_ROWS, int(bm))
        ys[bm] = G.gpu_gemm(dm, x, xdt)
    assert np.array_equal(ys["128"], ys["256"])
    # against the oracle fed the rounding of the weights the kernel declares (the gate against exact
    # binary32 weights is a statistical one for bf16 and is held by the other prefill tests)
    asfed = orc.linear(mat, orc.widen(x, xdt), "f64", weight_round=xdt)
    assert G.err_g2(ys["128"], asfed) <= 2e-5


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
@pytest.mark.parametrize("xdt", ["bf16", "f16"])
@pytest.mark.parametrize("N,K,M", [(512, 2048, 17), (256, 4096, 40), (768, 1024, 128), (256, 512, 100)])
def test_small_batch_both_paths(fmt, xdt, N, K, M, options):
    """16 < M <= 128 runs either on the matrix cores (M padded to 128 rows) or as ceil(M / 32) passes
    of the streaming kernels over row blocks of x (the 17..32-row instance, then one for the rest),
    whichever the dispatcher estimates cheaper.  Both
    are forced in turn; each against the oracle with the weights as that path feeds them (matrix
    cores: rounded to the type of x; streaming: exact), and the free choice equals one of them."""
    mat = make(fmt, N, K, 9)
    x = acts(M, K, xdt, M + 2)
    dm = B.upload(mat, native=True)
    ys = {}
    for path, fed in (("stream", None), ("mfma", xdt)):
        print(f"small batch via {path}: {fmt} N={N} K={K} M={M} x={xdt}", flush=True)
        options(B.OPT_SMALL_BATCH_PATH, FORCE[path])
        ys[path] = G.gpu_gemm(dm, x, xdt)
        asfed = orc.linear(mat, orc.widen(x, xdt), "f64", weight_round=fed)
        assert G.err_g2(ys[path], asfed) <= 2e-5, path
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_AUTO)
    free = G.gpu_gemm(dm, x, xdt)
    assert np.array_equal(free, ys["stream"]) or np.array_equal(free, ys["mfma"])
    # fp16 output as well (the row blocks of y are addressed in its element size)
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_STREAM)
    y16 = G.gpu_gemm(dm, x, xdt, B.F16)
    back = orc.widen(y16, "f16").astype(np.float64)
    assert np.abs(back - ys["stream"]).max() <= 2.0 ** -10 * np.abs(ys["stream"]).max()


def wide_range_rows(M, K, seed):
    """bf16 activation rows whose magnitudes leave what fp16 holds (|x| up to 65504, exact down to 2^-17):
    row m follows pattern m % 6 - the whole row at 7e4, the whole row at 1e-8, N(0, 1) with 1 % of the
    entries at +-7e4, N(0, 1) with 1 % of the entries at 1e-8 scale, the first half of the columns at 7e4
    and the second at 1e-8, and squared-ReLU values max(300 g, 0)^2 (the input of W'_v in Eq. "channel
    mixing o": many exact zeros, values up to 1e6)."""
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((M, K))
    for m in range(M):
        p = m % 6
        if p == 0:
            g[m] *= 7e4
        elif p == 1:
            g[m] *= 1e-8
        elif p == 2:
            pick = rng.random(K) < 0.01
            g[m, pick] = np.sign(g[m, pick]) * 7e4
        elif p == 3:
            pick = rng.random(K) < 0.01
            g[m, pick] *= 1e-8
        elif p == 4:
            g[m, : K // 2] *= 7e4
            g[m, K // 2:] *= 1e-8
        else:
            g[m] = np.maximum(300.0 * g[m], 0.0) ** 2
    return synth.f32_to_bf16_bits(g.astype(np.float32))


def rowwise_g2(y, ref):
    return max(G.err_g2(y[m:m + 1], ref[m:m + 1]) for m in range(y.shape[0]))


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
@pytest.mark.parametrize("M", [1, 6, 16, 32, 48])
def test_bf16_activations_of_any_magnitude(fmt, M, options, stretches):
    """Every finite bf16 activation is in contract.  The streaming kernels multiply fp16 operands: they
    must bring the activations into fp16's range with exact scales, so that a row of tiny values, a
    row of huge ones and rows that mix both all come out as the oracle computes them - row by row,
    since the rows of a batch are independent requests.  M = 48 runs both ways the dispatcher has
    for it (two streaming passes; the matrix cores, which multiply bf16 directly)."""
    N, K = 512, 1024
    mat = make(fmt, N, K, 21)
    dm = B.upload(mat, native=True)
    if M == 1:
        xs = [wide_range_rows(6, K, 50)[p:p + 1] for p in range(6)]        # each pattern as a call of its own
    else:
        xs = [wide_range_rows(M, K, 50 + M)]
    for path in (("stream", "mfma") if M > 16 else ("stream",)):
        options(B.OPT_SMALL_BATCH_PATH, FORCE[path])
        for x in xs:
            print(f"bf16 range {fmt} M={M} via {path}", flush=True)
            y = G.gpu_gemm(dm, x, "bf16")
            assert np.all(np.isfinite(y))
            ref = orc.linear(mat, orc.widen(x, "bf16"), "f64", weight_round="bf16" if path == "mfma" else None)
            assert rowwise_g2(y, ref) <= 2e-5, (path, rowwise_g2(y, ref))


@pytest.mark.parametrize("fmt", ["sq", "vq6", "vq8"])
def test_bf16_activations_of_any_magnitude_grouped_batch1(fmt):
    """The same through the batch-1 kernel that gives a wavefront a whole row tile (launches of 2048 row
    tiles and more; the test above runs the split-K kernel)."""
    N, K = 32768, 512
    mat = make(fmt, N, K, 22)
    dm = B.upload(mat, native=True)
    for p in range(6):
        print(f"bf16 range grouped {fmt} pattern {p}", flush=True)
        x = wide_range_rows(6, K, 60)[p:p + 1]
        y = G.gpu_gemm(dm, x, "bf16")
        ref = orc.linear(mat, orc.widen(x, "bf16"), "f64")
        # 1e-4, not 2e-5: with a few entries 7e4 times the rest (pattern 2) an SQ group's sum q.x and its
        # z * sum(x) are each 2^-24-accurate relative to 7e4 * 7 while their difference, the group's
        # contribution, is several times smaller; the scale of the activations plays no part in that
        assert G.err_g2(y, ref) <= 1e-4, p


@pytest.mark.parametrize("M", [17, 50, 128])
def test_small_batch_rows_not_multiple_of_256(M):
    """A native-layout matrix whose N is not a multiple of 256 has no matrix-core tiles; up to M = 128
    it runs as passes of the streaming kernels (exact weights), together with ordinary matrices of
    the same call."""
    torch = G.torch_()
    mats = [make("sq", 48, 768, 11), make("vq6", 256, 768, 12), make("sq", 400, 512, 13)]
    xs = [acts(M, m.K, "bf16", M + i) for i, m in enumerate(mats)]
    dms = [B.upload(m, native=True) for m in mats]
    xd = [G.to_dev_bits(x) for x in xs]
    ys = [torch.zeros((M, m.N), dtype=torch.float32, device="cuda") for m in mats]
    print(f"small batch, ragged N, M={M}", flush=True)
    B.rwkvq_linear_dispatch(B.DispatchTable([d.desc() for d in dms], xd, ys), M, B.BF16, B.F32)
    torch.cuda.synchronize()
    for i, (m, x, y) in enumerate(zip(mats, xs, ys)):
        exact = orc.linear(m, orc.widen(x, "bf16"), "f64")
        got = y.cpu().numpy().astype(np.float64)
        if m.N % 256:
            assert G.err_g2(got, exact) <= 2e-5, i          # streaming passes: exact weights
        elif G.err_g2(got, exact) > 2e-5:                   # the dispatcher chose the matrix cores for this one
            G.check_outputs(got, m, x, "bf16", fed="bf16")


def test_dispatch_randomized_batches_and_paths(options):
    """Seeded sweep over batch sizes 1..300, call compositions and the small-batch override: every
    output against the oracle with the weights as the reported path feeds them (rwkvq_linear_dispatch_plan:
    exact for the streaming kernels and the reference kernel, rounded to the type of x on the matrix
    cores).  Catches row-block offsets, ragged last passes (M = 33: 32 rows + 1) and mixed calls."""
    torch = G.torch_()
    rng = np.random.default_rng(4242)
    shapes = [(256, 512), (512, 256), (256, 1024), (768, 768), (48, 512), (1024, 256)]
    for case in range(36):
        M = int(rng.choice([1, 2, 5, 16, 17, 31, 32, 33, 47, 64, 65, 96, 100, 128, 129, 200, 300]))
        xdt = ("f16", "bf16")[case % 2]
        n = int(rng.integers(1, 4))
        mats = []
        for j in range(n):
            N, K = shapes[int(rng.integers(0, len(shapes)))]
            fmt = ("sq", "vq6", "vq8")[int(rng.integers(0, 3))]
            if fmt != "sq" and N % 256:
                N = 256
            mats.append(make(fmt, N, K, 100 + 7 * case + j))
        override = (None, "stream", "mfma")[int(rng.integers(0, 3))]
        options(B.OPT_SMALL_BATCH_PATH, FORCE[override])
        dms = [B.upload(m, native=True) for m in mats]
        descs = [d.desc() for d in dms]
        xs = [acts(M, m.K, xdt, 1000 + case * 10 + j) for j, m in enumerate(mats)]
        ys = [torch.full((M, m.N), 7.0, dtype=torch.float32, device="cuda") for m in mats]
        paths = B.rwkvq_linear_dispatch_plan(descs, M)
        print(f"randomized case {case}: M={M} x={xdt} override={override} "
              f"mats={[(m.kind, m.N, m.K) for m in mats]} paths={paths}", flush=True)
        B.rwkvq_linear_dispatch(B.DispatchTable(descs, [G.to_dev_bits(x) for x in xs], ys), M, B.DTYPES[xdt], B.F32)
        torch.cuda.synchronize()
        for m, x, y, p in zip(mats, xs, ys, paths):
            fed = xdt if p == B.PATH_MATRIX_CORES else None
            ref = orc.linear(m, orc.widen(x, xdt), "f64", weight_round=fed)
            assert G.err_g2(y.cpu().numpy().astype(np.float64), ref) <= 2e-5, (case, m.kind, m.N, m.K, p)
