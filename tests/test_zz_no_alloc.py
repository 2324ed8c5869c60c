"""The allocation-free entry point, wash_consensus_sqdist_noalloc, through the C ABI: same result as
wash_consensus_sqdist bit for bit (the bar for this fixed-shape fp64 reduction), within 1e-10 of the
oracle, on two calls in a row, the second on a smaller input (the fixed scratch keeps the first call's
partial sums), with no device allocation made by the calls."""
import ctypes

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def wash():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_17517_amd as w
    return w


def _raw_noalloc(wash, d, a, b, out):
    N, P = d.shape
    stream = torch.cuda.current_stream().cuda_stream
    rc = wash.binding.raw.wash_consensus_sqdist_noalloc(d.data_ptr(), N, P, a, b, out.data_ptr(), stream)
    assert rc == 0, wash.binding.raw.wash_last_error_detail()


def test_noalloc_matches_the_allocating_entry_point_twice_in_a_row(wash):
    rng = np.random.default_rng(5)
    big = (rng.standard_normal((8, 3_000_017)) * 0.02).astype(np.float32)       # 2930 blocks: most of the scratch
    small = (rng.standard_normal((3, 70_001)) * 0.5).astype(np.float32)         # 69 blocks, fewer models
    d_big, d_small = torch.from_numpy(big).cuda(), torch.from_numpy(small).cuda()
    out_big = torch.full((8,), -1.0, dtype=torch.float64, device="cuda")
    out_small = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    # the reference entry point first (it may allocate its scratch), so that the counters below see the new calls only
    ref_big = wash.wash_consensus_sqdist(d_big).cpu().numpy()
    ref_small = wash.wash_consensus_sqdist(d_small, 11, 65_000).cpu().numpy()
    torch.cuda.synchronize()
    out_again = torch.full((8,), -1.0, dtype=torch.float64, device="cuda")
    out_empty = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    print("noalloc: first call, N=8 P=3000017", flush=True)
    _raw_noalloc(wash, d_big, 0, 3_000_017, out_big)          # also looks up the array's address on this device
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    print("noalloc: second call, N=3 P=70001 slice [11, 65000)", flush=True)
    _raw_noalloc(wash, d_small, 11, 65_000, out_small)
    print("noalloc: third and fourth call, the large input again and an empty slice", flush=True)
    _raw_noalloc(wash, d_big, 0, 3_000_017, out_again)
    _raw_noalloc(wash, d_small, 5, 5, out_empty)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 >= free0                                     # the calls took no device memory
    assert torch.equal(out_empty.cpu(), torch.zeros(3, dtype=torch.float64))
    assert np.array_equal(out_big.cpu().numpy(), ref_big)
    assert np.array_equal(out_small.cpu().numpy(), ref_small)
    assert np.array_equal(out_again.cpu().numpy(), ref_big)
    assert np.allclose(ref_big, oracle.consensus_sqdist(big), rtol=1e-10, atol=0)
    assert np.allclose(ref_small, oracle.consensus_sqdist(small, 11, 65_000), rtol=1e-10, atol=0)


def test_noalloc_rejects_what_the_fixed_scratch_does_not_cover(wash):
    d = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    raw = wash.binding.raw
    assert raw.wash_consensus_sqdist_noalloc(d.data_ptr(), 33, 100, 0, 100, out.data_ptr(), None) == -1
    assert b"1..32" in raw.wash_last_error_detail()
    assert raw.wash_consensus_sqdist_noalloc(d.data_ptr(), 2, (1 << 40) + 1, 0, 100, out.data_ptr(), None) == -1
    assert b"2^40" in raw.wash_last_error_detail()
    assert raw.wash_consensus_sqdist_noalloc(d.data_ptr(), 2, 100, 50, 20, out.data_ptr(), None) == -1
    assert raw.wash_consensus_sqdist_noalloc(d.data_ptr(), 2, 100, 0, 101, out.data_ptr(), None) == -1
    assert raw.wash_consensus_sqdist_noalloc(None, 2, 100, 0, 100, out.data_ptr(), None) == -1
    assert raw.wash_consensus_sqdist_noalloc(d.data_ptr(), 2, 100, 0, 100, None, None) == -1
    with pytest.raises(TypeError):
        wash.wash_consensus_sqdist_noalloc(d, torch.zeros(3, dtype=torch.float64, device="cuda"))
    got = wash.wash_consensus_sqdist_noalloc(d + 1.0, out)      # identical rows: zero distance
    assert got.data_ptr() == out.data_ptr() and torch.equal(out.cpu(), torch.zeros(2, dtype=torch.float64))
