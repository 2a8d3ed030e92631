"""The benchmark's yardstick kernels (bench_yardsticks.hip, a library of its own beside bench.py) do what their
comments say: the figures bench.py derives from them rest on the bytes they move."""
import ctypes as C
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ys():
    torch.cuda.init()
    lib = C.CDLL(os.path.join(ROOT, "libbench_yardsticks.so"))
    lib.ys_sweep.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.ys_update_pattern.argtypes = [C.c_void_p] * 5 + [C.c_uint64, C.c_int32, C.c_void_p]
    lib.ys_link.argtypes = [C.c_void_p] * 4 + [C.c_size_t, C.c_int32, C.POINTER(C.c_double)]
    lib.ys_last_error.restype = C.c_char_p
    return lib


@pytest.mark.parametrize("n", [8, 1024, 1028, 300_004])
def test_sweeps(ys, n):
    x = torch.full((n,), 3.0, dtype=torch.float32, device="cuda:0")
    assert ys.ys_sweep(0, x.data_ptr(), 4 * n, None) == 0
    torch.cuda.synchronize()
    assert bool((x == 3.0).all())
    assert ys.ys_sweep(2, x.data_ptr(), 4 * n, None) == 0
    torch.cuda.synchronize()
    h = x.cpu().numpy()
    assert (h[:-4] == 1.5).all() and (h[-4:] == 3.0).all()          # the last 16 bytes are left alone
    assert ys.ys_sweep(1, x.data_ptr(), 4 * n, None) == 0
    torch.cuda.synchronize()
    h = x.cpu().numpy()
    i = np.arange(n - 4) // 4
    assert np.array_equal(h[:-4], (i % 1024) + 0.25 * (np.arange(n - 4) % 4)) and (h[-4:] == 3.0).all()
    assert ys.ys_sweep(3, x.data_ptr(), 4 * n, None) < 0 and b"kind" in ys.ys_last_error()


@pytest.mark.parametrize("n,T", [(4096, 0), (10_000, 0), (8192, 1024), (20_000, 8192)])
def test_update_pattern_touches_every_element_once(ys, n, T):
    d = "cuda:0"
    g = torch.arange(n, dtype=torch.int32, device=d).to(torch.int16)
    h = torch.zeros(n, dtype=torch.int16, device=d)
    if T:
        nt = -(-n // T)
        st = torch.full((nt * 3 * T,), 4.0, dtype=torch.float32, device=d)
        assert ys.ys_update_pattern(st.data_ptr(), None, None, g.data_ptr(), h.data_ptr(), n, T, None) == 0
        torch.cuda.synchronize()
        a = st.cpu().numpy().reshape(nt, 3, T)
        for j in range(3):
            flat = a[:, j, :].reshape(-1)
            assert (flat[:n] == 2.0).all() and (flat[n:] == 4.0).all()
    else:
        p, m, v = (torch.full((n,), 4.0, dtype=torch.float32, device=d) for _ in range(3))
        assert ys.ys_update_pattern(p.data_ptr(), m.data_ptr(), v.data_ptr(), g.data_ptr(), h.data_ptr(), n, 0,
                                    None) == 0
        torch.cuda.synchronize()
        assert all(bool((x == 2.0).all()) for x in (p, m, v))
    assert np.array_equal(h.cpu().numpy(), g.cpu().numpy() ^ 1)


def test_link_copies(ys):
    n = 1 << 20
    a = torch.arange(n, dtype=torch.float32).pin_memory()
    b = torch.zeros(n, dtype=torch.float32).pin_memory()
    da = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    db = torch.full((n,), 7.0, dtype=torch.float32, device="cuda:0")
    sec = (C.c_double * 3)()
    assert ys.ys_link(a.data_ptr(), da.data_ptr(), db.data_ptr(), b.data_ptr(), 4 * n, 2, sec) == 0
    torch.cuda.synchronize()
    assert torch.equal(da.cpu(), a) and bool((b == 7.0).all())
    assert all(0.0 < s < 1.0 for s in sec)
