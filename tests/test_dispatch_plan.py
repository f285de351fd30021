"""Host logic of the dispatcher (no GPU): which kernels a call's matrices are routed to, from M and
the sizes and layouts alone.  rwkvq_linear_dispatch_plan runs the same decision code as the dispatch
itself and touches no device."""
import pytest

from paper_2505_03803_amd import binding as B

FAKE = 0x7F0000000000        # aligned, never dereferenced


def sq(N, K, layout=B.NATIVE):
    zeros = FAKE if layout == B.CANONICAL else None
    return B.rwkvq_matrix(B.SQ, layout, N, K, 3, 128, 0, 0, 0, 0, FAKE, FAKE, zeros, None)


def vq(N, K, kbits=6, layout=B.NATIVE):
    return B.rwkvq_matrix(B.VQ, layout, N, K, 0, 0, 2, kbits, 256, 256, FAKE, None, None, FAKE)


def layer_7b():
    d, f = 4096, 14336
    return [sq(d, d), vq(d, d), sq(d, d), vq(d, d), sq(d, d), vq(f, d), sq(d, f), vq(d, d, 8)]


@pytest.fixture(autouse=True)
def no_override(options):
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_AUTO)


def test_batch_up_to_16_streams():
    for M in (1, 2, 16):
        assert B.rwkvq_linear_dispatch_plan(layer_7b(), M) == [B.PATH_STREAM] * 8


def test_large_batch_takes_the_matrix_cores():
    for M in (129, 2048, 4096):
        assert B.rwkvq_linear_dispatch_plan(layer_7b(), M) == [B.PATH_MATRIX_CORES] * 8


def test_canonical_layout_takes_the_reference_kernel_whatever_m():
    mats = [sq(256, 512, B.CANONICAL), vq(256, 512, 6, B.CANONICAL), sq(256, 512)]
    assert B.rwkvq_linear_dispatch_plan(mats, 1) == [B.PATH_REFERENCE, B.PATH_REFERENCE, B.PATH_STREAM]
    assert B.rwkvq_linear_dispatch_plan(mats, 300) == [B.PATH_REFERENCE, B.PATH_REFERENCE, B.PATH_MATRIX_CORES]


def test_small_batch_is_decided_by_the_size_of_the_call():
    one = [sq(4096, 4096)]
    stack = layer_7b() * 32
    # one matrix: 16 workgroups on the matrix cores whatever M; passes of the streaming kernels win up to M = 96
    for M, want in ((17, B.PATH_STREAM_PASSES), (32, B.PATH_STREAM_PASSES), (64, B.PATH_STREAM_PASSES),
                    (96, B.PATH_STREAM_PASSES), (128, B.PATH_MATRIX_CORES)):
        assert B.rwkvq_linear_dispatch_plan(one, M) == [want], M
    # the whole stack fills the device either way: two passes at most
    for M, want in ((17, B.PATH_STREAM_PASSES), (32, B.PATH_STREAM_PASSES), (48, B.PATH_STREAM_PASSES),
                    (64, B.PATH_STREAM_PASSES), (96, B.PATH_MATRIX_CORES), (128, B.PATH_MATRIX_CORES)):
        assert set(B.rwkvq_linear_dispatch_plan(stack, M)) == {want}, M
    # a short K makes the matrix-core workgroups short: they win early
    assert B.rwkvq_linear_dispatch_plan([sq(256, 512)], 64) == [B.PATH_MATRIX_CORES]


def test_rows_not_a_multiple_of_256_have_no_matrix_core_tiles():
    mats = [sq(48, 768), sq(256, 768)]
    assert B.rwkvq_linear_dispatch_plan(mats, 16) == [B.PATH_STREAM, B.PATH_STREAM]
    assert B.rwkvq_linear_dispatch_plan(mats, 100)[0] == B.PATH_STREAM_PASSES
    assert B.rwkvq_linear_dispatch_plan(mats, 129) == [B.PATH_REFERENCE, B.PATH_MATRIX_CORES]


def test_rows_longer_than_the_streaming_kernels_hold():
    long_k = [sq(256, 20480 + 256)]
    assert B.rwkvq_linear_dispatch_plan(long_k, 1) == [B.PATH_REFERENCE]
    assert B.rwkvq_linear_dispatch_plan(long_k, 64) == [B.PATH_MATRIX_CORES]
    assert B.rwkvq_linear_dispatch_plan([sq(48, 20480 + 256)], 64) == [B.PATH_REFERENCE]


def test_forced_path(options):
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_MATRIX_CORES)
    assert B.rwkvq_linear_dispatch_plan([sq(4096, 4096)], 32) == [B.PATH_MATRIX_CORES]
    options(B.OPT_SMALL_BATCH_PATH, B.SMALL_BATCH_STREAM)
    assert B.rwkvq_linear_dispatch_plan([sq(256, 512)], 128) == [B.PATH_STREAM_PASSES]
    assert B.rwkvq_linear_dispatch_plan([sq(256, 512)], 129) == [B.PATH_MATRIX_CORES]      # beyond 128: no choice


def test_estimate_constants_are_settable(options):
    """The estimate's constants are one machine's; another machine's replace them through rwkvq_set_option."""
    one = [sq(4096, 4096)]
    assert B.rwkvq_linear_dispatch_plan(one, 64) == [B.PATH_STREAM_PASSES]
    options(B.OPT_STREAM_WIDE_MIN_US, 200)                       # a machine whose streaming passes start slowly
    assert B.rwkvq_linear_dispatch_plan(one, 64) == [B.PATH_MATRIX_CORES]
    options(B.OPT_STREAM_WIDE_MIN_US, 0)                         # 0 = the default again
    assert B.rwkvq_get_option(B.OPT_STREAM_WIDE_MIN_US) == 24
    assert B.rwkvq_linear_dispatch_plan(one, 64) == [B.PATH_STREAM_PASSES]
    options(B.OPT_MFMA_KSTEP_NS, 100)                            # much faster matrix-core steps
    assert B.rwkvq_linear_dispatch_plan(one, 64) == [B.PATH_MATRIX_CORES]


def test_option_rejects():
    assert B.rwkvq_set_option(99, 1, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_set_option(-1, 1, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_set_option(B.OPT_SMALL_BATCH_PATH, 3, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_set_option(B.OPT_PREFILL_TILE_ROWS, 64, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_set_option(B.OPT_STREAM_WIDE_GBPS, -5, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_set_option(B.OPT_STREAM_TWO_PASS_MIN_WGS, 1000001, check=False) == B.ERR_UNSUPPORTED
    assert B.rwkvq_get_option(B.OPT_STREAM_TWO_PASS_MIN_WGS) == 2048
    assert B.rwkvq_get_option(B.OPT_STREAM_SPLIT_MAX_WORK) == 65536
    assert B.lib().rwkvq_get_option(0, None) == B.ERR_NULL


def test_plan_rejects():
    L = B.lib()
    from ctypes import c_int32
    out = (c_int32 * 1)()
    good = (B.rwkvq_matrix * 1)(sq(256, 512))
    assert L.rwkvq_linear_dispatch_plan(None, 1, 1, out) == B.ERR_NULL
    assert L.rwkvq_linear_dispatch_plan(good, 1, 1, None) == B.ERR_NULL
    assert L.rwkvq_linear_dispatch_plan(good, 0, 1, out) == B.ERR_SHAPE
    assert L.rwkvq_linear_dispatch_plan(good, 1, 0, out) == B.ERR_SHAPE
    bad = (B.rwkvq_matrix * 1)(sq(250, 512))
    assert L.rwkvq_linear_dispatch_plan(bad, 1, 1, out) == B.ERR_SHAPE
