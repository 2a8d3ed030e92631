"""mlpo_grad_unscale_norm_static - the gradient pass for callers that cannot allocate - against
mlpo_grad_unscale_norm on the same gradients: the 16-byte record must be the same bit for bit (same kernels, same
order of summation; the only difference is where the per-workgroup partial sums live), on two calls in a row, the
second with a smaller input, so that whatever the first call left in the library's static array is shown not to
matter."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, dev, to_dev_u16  # noqa: E402


def record(t):
    h = t.cpu().numpy()
    return h.view(np.uint32).tolist()


def gradient_table(sizes, seed, loss_scale, offset):
    """Subgroups as slices of one flat gradient buffer that starts `offset` elements into an allocation, so that the
    slices have every alignment."""
    total = sum(sizes)
    host = np.empty(total, np.uint16)
    W.fill_grad_bf16(host, seed, 0, 0, 1e-3, loss_scale, threads=8)
    flat = torch.zeros(total + offset, dtype=torch.int16, device=dev())
    flat[offset:] = to_dev_u16(host)
    sgs, lo = [], 0
    for n in sizes:
        g = flat[offset + lo:offset + lo + n]
        sgs.append(B.SubgroupC(None, None, None, g.data_ptr(), None, n, B.TIER_HBM, 0, B.HALF_BF16, 0))
        lo += n
    return B.SubgroupTable(sgs), flat, host


def test_static_entry_matches_the_workspace_entry_twice(oracle):
    scratch = Scratch()
    out_static = torch.zeros(4, dtype=torch.float32, device=dev())
    st = torch.cuda.current_stream()
    # first call: 16 subgroups of 1.1 M gradients (several rounds of the persistent grid, ragged tails, odd
    # alignments), loss scale 1024 with clipping; second call: three small subgroups, one of them empty, no clipping
    calls = [([1_100_003] * 15 + [77_777], 5, 1024.0, 0.25, 3),
             ([4099, 0, 513], 6, 1.0, 0.0, 1)]
    for sizes, seed, scale, max_norm, offset in calls:
        table, flat, host = gradient_table(sizes, seed, scale, offset)
        inv = float(np.float32(1.0 / scale))
        print(f"static entry: {len(sizes)} subgroups, {sum(sizes)} gradients", flush=True)
        B.mlpo_grad_unscale_norm(table, inv, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
        B.mlpo_grad_unscale_norm_static(table, inv, max_norm, out_static, st)
        torch.cuda.synchronize()
        assert record(out_static) == record(scratch.scalars), (record(out_static), record(scratch.scalars))
        # and both agree with the oracle to the bar of the gradient pass: flag exact, norm within 1e-5
        sumsq, flag = oracle.grad_stats(host, inv)
        norm_o, coef_o, gmul_o = oracle.norm_finish(sumsq, inv, max_norm)
        got = out_static.cpu().numpy()
        assert int(got[3:4].view(np.uint32)[0]) == flag == 0
        assert abs(float(got[0]) - float(norm_o)) <= 1e-5 * float(norm_o)
        assert float(got[2]) == float(gmul_o)
    # a non-finite gradient in the second, smaller input: the flag comes out of the static array as well
    table, flat, host = gradient_table([4099, 0, 513], 6, 1.0, 1)
    flat[1 + 4099 + 500] = 0x7F80
    B.mlpo_grad_unscale_norm_static(table, 1.0, 0.0, out_static, st)
    B.mlpo_grad_unscale_norm(table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
    torch.cuda.synchronize()
    assert record(out_static)[3] == 1 and record(scratch.scalars)[3] == 1


def test_static_entry_rejects_what_exceeds_its_limits():
    out = torch.zeros(4, dtype=torch.float32, device=dev())
    g = torch.zeros(8, dtype=torch.int16, device=dev())
    one = B.SubgroupC(None, None, None, g.data_ptr(), None, 8, B.TIER_HBM, 0, B.HALF_BF16, 0)
    with pytest.raises(B.MlpoError) as e:
        B.mlpo_grad_unscale_norm_static([one] * 1025, 1.0, 0.0, out)
    assert e.value.code == B.MLPO_EINVAL and "at most 1024" in str(e.value)
    huge = B.SubgroupC(None, None, None, g.data_ptr(), None, (1 << 40) + 8, B.TIER_HBM, 0, B.HALF_BF16, 0)
    with pytest.raises(B.MlpoError) as e:
        B.mlpo_grad_unscale_norm_static([huge], 1.0, 0.0, out)
    assert e.value.code == B.MLPO_EINVAL and "at most" in str(e.value)
    B.mlpo_grad_unscale_norm_static([], 1.0, 0.0, out)          # an empty table is a norm of zero
    torch.cuda.synchronize()
    assert out.cpu().numpy()[0] == 0.0
