"""rwkvq_proxy_static (the proxy call for callers that cannot allocate: its bitmaps live in a device
array inside the library) against rwkvq_proxy with a caller's workspace: the same kernels, so the
same bits, on two calls in a row, the second with a smaller input (the array keeps the first call's
contents and must be cleared by the call itself).  Collected last: the file name sorts after the
other test files."""
import ctypes

import numpy as np
import pytest

from paper_2505_03803_amd import synth


def test_static_entry_point_rejects_without_gpu():
    from paper_2505_03803_amd import binding as B
    L = B.lib()
    FAKE = 0x10000
    n = B_MAX = 256
    ws = (ctypes.c_void_p * (n + 1))(*([FAKE] * (n + 1)))
    Ns = (ctypes.c_int * (n + 1))(*([16] * (n + 1)))
    Ks = (ctypes.c_int * (n + 1))(*([16] * (n + 1)))
    call = lambda **kw: L.rwkvq_proxy_static(kw.get("ws", ws), kw.get("Ns", Ns), kw.get("Ks", Ks), kw.get("n", 1),
                                             kw.get("dt", B.BF16), kw.get("terms", 5), 1.5, 50.0,
                                             kw.get("out", FAKE), kw.get("phi", FAKE), None)
    assert call(n=B_MAX + 1) == B.ERR_SHAPE          # beyond the array's capacity
    assert call(n=0) == B.ERR_SHAPE
    assert call(out=None) == B.ERR_NULL
    assert call(phi=None) == B.ERR_NULL
    assert call(dt=B.F32) == B.ERR_UNSUPPORTED
    assert call(terms=9) == B.ERR_UNSUPPORTED
    assert call(out=FAKE + 8) == B.ERR_ALIGN


@pytest.mark.gpu
def test_static_equals_workspace_call_twice():
    import torch
    from paper_2505_03803_amd import binding as B
    rng = np.random.default_rng(11)

    def both(shapes, dtype):
        mats = [synth.gen_dense_weights(rng, N, K, dtype, outlier_fraction=1e-3 * (i % 2)) for i, (N, K) in enumerate(shapes)]
        dev = [torch.from_numpy(m.view(np.int16)).cuda() for m in mats]
        n = len(dev)
        table = B.ProxyTable(dev, shapes)
        wsp = torch.empty(B.rwkvq_proxy_workspace_bytes(n) // 4, dtype=torch.int32, device="cuda")
        o1 = torch.zeros(2 * n, dtype=torch.float64, device="cuda"); f1 = torch.full((n + 3,), -7, dtype=torch.int32, device="cuda")
        o2 = torch.zeros(2 * n, dtype=torch.float64, device="cuda"); f2 = torch.full((n + 3,), -7, dtype=torch.int32, device="cuda")
        print(f"proxy_static n={n} dtype={dtype} shapes[0]={shapes[0]}", flush=True)
        B.rwkvq_proxy(table, B.DTYPES[dtype], 5, 9.0, 1e12, wsp, o1, f1)
        B.rwkvq_proxy_static(table, B.DTYPES[dtype], 5, 9.0, 1e12, o2, f2)
        torch.cuda.synchronize()
        a, b = o1.cpu().numpy(), o2.cpu().numpy()
        assert np.array_equal(a.view(np.uint64), b.view(np.uint64)), (a, b)
        assert torch.equal(f1, f2)
        assert np.all(np.isfinite(a)) and np.all(a[0::2] > 0.0)
        return mats, a

    # first call: 70 matrices (two launches of the grouped kernels, 560 KiB of the array), wide value sets
    shapes1 = [(64 + 16 * (i % 5), 96 + 8 * (i % 7)) for i in range(69)] + [(1024, 1536)]
    both(shapes1, "bf16")
    # second call, smaller: 3 matrices with few distinct values; bits left over from the first call
    # would add values that are not there and change every sum
    shapes2 = [(32, 64), (7, 33), (16, 16)]
    mats, got = both(shapes2, "f16")
    from oracle import proxy_oracle as PO
    for i, m in enumerate(mats):
        ePc, ePf = PO.proxies(PO.widen16(m, "f16"))
        assert got[2 * i] == pytest.approx(ePc, rel=1e-9) and got[2 * i + 1] == pytest.approx(ePf, rel=1e-9)
