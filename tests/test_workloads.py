"""The seeded input generator: slices regenerate identically, shapes match the five workloads."""
import numpy as np

from paper_2509_02480_amd import workloads as W


def test_slices_regenerate_identically():
    n = 3 * W.CHUNK + 1234
    full = np.empty(n, np.float32)
    W.fill_normal_f32(full, 3, W.T_PARAM, 0, 0, 0.02)
    for start, cnt in ((0, 10), (W.CHUNK - 5, 20), (2 * W.CHUNK + 7, W.CHUNK + 100), (n - 1, 1)):
        part = np.empty(cnt, np.float32)
        W.fill_normal_f32(part, 3, W.T_PARAM, 0, start, 0.02, threads=4)
        assert np.array_equal(part, full[start:start + cnt])
    g = np.empty(n, np.uint16)
    W.fill_grad_bf16(g, 3, 2, 0, 1e-3, 1024.0, threads=4)
    g2 = np.empty(1000, np.uint16)
    W.fill_grad_bf16(g2, 3, 2, W.CHUNK - 500, 1e-3, 1024.0)
    assert np.array_equal(g2, g[W.CHUNK - 500:W.CHUNK + 500])
    other = np.empty(1000, np.uint16)
    W.fill_grad_bf16(other, 3, 3, W.CHUNK - 500, 1e-3, 1024.0)
    assert not np.array_equal(other, g2)


def test_distributions():
    p = np.empty(1 << 20, np.float32)
    W.fill_normal_f32(p, 0, W.T_PARAM, 0, 0, 0.02)
    assert abs(p.std() / 0.02 - 1) < 0.01 and abs(p.mean()) < 1e-4
    g = np.empty(1 << 20, np.uint16)
    W.fill_grad_bf16(g, 0, 0, 0, 1e-3, 1024.0)
    gv = (g.astype(np.uint32) << 16).view(np.float32)
    assert abs(gv.std() / 1.024 - 1) < 0.01 and np.isfinite(gv).all()


def test_workload_shapes():
    assert W.C1.n_total == 1_048_576 and W.C1.n_host == 0
    assert W.C2.n_total == 125_000_000 and W.C2.sub_elems % 4 == 0 and W.C2.sub_elems % 8 != 0
    assert W.C3.n_total == 1_300_000_000 and W.C3.n_host == 13
    assert (W.C4.n_total, W.C4.n_host) == (7_000_000_000, 18)
    assert (W.C5.n_total, W.C5.n_host) == (8_750_000_000, 25) and W.C5.inv_scale == 2.0 ** -16
    assert [s for s in range(10) if W.C2.injects(s)] == [4]
    assert 0 <= W.C2.inject_index(4) < W.C2.n_total
    half = W.C4.scaled_down(5)
    assert half.n_sub == 7 and half.n_host == 4 and half.sub_elems == W.C4.sub_elems
    assert [W.C4.tier(k) for k in (0, 17, 18, 34)] == [1, 1, 0, 0]
