"""The hot path inside a captured HIP graph: after a first eager call (which builds the cached
segment table) the entry points only launch kernels on the caller's stream, so a step can be
captured and replayed.  Every replay is checked against eager execution, with eager work and
synchronisation between the replays."""
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


@pytest.mark.parametrize("stream", ["v1", "gap"])
def test_step_replays_in_a_graph(wash, stream):
    shuffle = wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap
    N, P = 5, 300_007
    rng = np.random.default_rng(0)
    host = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    segs = wash.SegmentList([(0, P // 2, 0.01), (P // 2, P - P // 2, 0.05)])
    segs_list = [(0, P // 2, 0.01), (P // 2, P - P // 2, 0.05)]

    pop = torch.from_numpy(host).cuda()
    mom = pop.clone()
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    out = torch.empty(P, dtype=torch.float32, device="cuda")
    dist = torch.empty(N, dtype=torch.float64, device="cuda")

    def step():
        shuffle(pop, mom, segs, 7, 3, cnt)
        wash.papa_ema(pop, 0.9)
        wash.wash_average(pop, out)
        wash.wash_consensus_sqdist(pop, 0, P, dist)

    # warm-up on a side stream (builds the cached table and the scratch buffer), then capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    pop.copy_(torch.from_numpy(host))
    mom.copy_(torch.from_numpy(host))
    cnt.zero_()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    # capture only records: nothing ran yet
    torch.cuda.synchronize()
    assert torch.equal(pop.cpu(), torch.from_numpy(host)) and int(cnt.item()) == 0

    ref, refm = host.copy(), host.copy()
    ref_cnt = 0
    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        ref_cnt += oracle.shuffle(ref, refm, segs_list, 7, 3, stream=stream)
        oracle.ema(ref, 0.9)
        assert np.array_equal(pop.cpu().numpy().view(np.uint32), ref.view(np.uint32)), replay
        assert np.array_equal(mom.cpu().numpy().view(np.uint32), refm.view(np.uint32)), replay
        assert int(cnt.item()) == ref_cnt
        assert np.array_equal(out.cpu().numpy(), oracle.average(ref))
        assert np.allclose(dist.cpu().numpy(), oracle.consensus_sqdist(ref), rtol=1e-10)
        # eager work between replays on other buffers must not disturb the graph's state
        other = torch.from_numpy(host).cuda()
        shuffle(other, None, segs, 1, replay)
        wash.wash_average(other)
        torch.cuda.synchronize()


@pytest.mark.parametrize("gap", [False, True])
def test_device_step_advances_across_replays(wash, gap):
    """wash_shuffle_device_step reads the step from device memory, so one captured launch replays as
    successive iterations of Alg. 1: fresh mask and permutations at every replay."""
    stream = "gap" if gap else "v1"
    N, P = 6, 200_003
    rng = np.random.default_rng(5)
    hosts = [(rng.standard_normal((N, P)) * 0.02).astype(np.float32) for _ in range(3)]
    segs_list = [(0, P // 3, 0.02), (P // 3, P - P // 3 - 1000, 0.004)]
    segs = wash.SegmentList(segs_list)
    empty = wash.SegmentList([(10, 100, 0.0)])
    bufs = [torch.from_numpy(h).cuda() for h in hosts]
    step = torch.full((1,), 40, dtype=torch.int64, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")

    # eager: step taken from the device word, advanced afterwards; with advance=False it stays
    refs = [h.copy() for h in hosts]
    ref_cnt = 0
    wash.wash_shuffle_device_step(bufs, segs, 9, step, advance=False, gap_stream=gap, selected_count=cnt)
    wash.wash_shuffle_device_step(bufs, segs, 9, step, advance=True, gap_stream=gap, selected_count=cnt)
    wash.wash_shuffle_device_step(bufs, empty, 9, step, advance=True, gap_stream=gap)     # nothing to shuffle: still advances
    torch.cuda.synchronize()
    assert int(step.item()) == 42
    for s_ in (40, 40):
        for r in refs:
            c = oracle.shuffle(r, None, segs_list, 9, s_, stream=stream)
        ref_cnt += c
    assert int(cnt.item()) == ref_cnt
    for b, r in zip(bufs, refs):
        assert np.array_equal(b.cpu().numpy().view(np.uint32), r.view(np.uint32))

    # captured once, replayed five times: steps 42 .. 46
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wash.wash_shuffle_device_step(bufs, segs, 9, step, advance=True, gap_stream=gap, selected_count=cnt)
    torch.cuda.synchronize()
    assert int(step.item()) == 42
    for replay in range(5):
        graph.replay()
        torch.cuda.synchronize()
        for r in refs:
            c = oracle.shuffle(r, None, segs_list, 9, 42 + replay, stream=stream)
        ref_cnt += c
        assert int(step.item()) == 43 + replay
        assert int(cnt.item()) == ref_cnt
        for b, r in zip(bufs, refs):
            assert np.array_equal(b.cpu().numpy().view(np.uint32), r.view(np.uint32)), replay
        other = torch.from_numpy(hosts[0]).cuda()                 # eager work between replays
        wash.wash_shuffle(other, None, segs, 1, replay)
        torch.cuda.synchronize()
    # the two-buffer entry point at the same step gives the same bits
    a, b = torch.from_numpy(hosts[0]).cuda(), torch.from_numpy(hosts[1]).cuda()
    c, d = a.clone(), b.clone()
    step.fill_(1234)
    wash.wash_shuffle_device_step([a, b], segs, 3, step, advance=False, gap_stream=gap)
    (wash.wash_shuffle_gap if gap else wash.wash_shuffle)(c, d, segs, 3, 1234)
    assert torch.equal(a, c) and torch.equal(b, d)


def test_table_of_a_captured_launch_survives_cache_eviction(wash):
    # the library caches 16 segment tables; a table that a captured launch refers to must outlive
    # any number of later segment lists, because every replay reads it again
    N, P = 4, 50_021
    rng = np.random.default_rng(9)
    host = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    segs_list = [(3, 20_000, 0.05), (25_000, 25_000, 0.01)]
    segs = wash.SegmentList(segs_list)
    pop = torch.from_numpy(host).cuda()
    step = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_shuffle_device_step([pop], segs, 2, step, advance=False)      # builds the table outside the capture
    torch.cuda.synchronize()
    pop.copy_(torch.from_numpy(host))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wash.wash_shuffle_device_step([pop], segs, 2, step, advance=True)
    ref = host.copy()
    for replay in range(3):
        other = torch.from_numpy(host).cuda()
        for k in range(20):                                                  # 20 new lists: evicts every unpinned table
            wash.wash_shuffle(other, None, [(k + 1 + 100 * replay, 1000 + k, 0.1)], 0, 0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        oracle.shuffle(ref, None, segs_list, 2, replay)
        assert np.array_equal(pop.cpu().numpy().view(np.uint32), ref.view(np.uint32)), replay


def test_captured_call_that_uses_both_kernels(wash):
    # a list with a dense segment (p = 0.6, streamed through LDS), a sparse one and ragged ends uses two
    # segment tables and two kernels per call; both tables must survive later lists, the step advances once
    N, P = 6, 90_011
    rng = np.random.default_rng(21)
    hosts = [(rng.standard_normal((N, P)) * 0.02).astype(np.float32) for _ in range(2)]
    segs_list = [(7, 40_000, 0.6), (40_007, 30_000, 0.003), (75_000, P - 75_000, 1.0)]
    segs = wash.SegmentList(segs_list)
    bufs = [torch.from_numpy(h).cuda() for h in hosts]
    step = torch.full((1,), 5, dtype=torch.int64, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    wash.wash_shuffle_device_step(bufs, segs, 77, step, advance=False, selected_count=cnt)   # builds both tables
    torch.cuda.synchronize()
    for b, h in zip(bufs, hosts):
        b.copy_(torch.from_numpy(h))
    cnt.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wash.wash_shuffle_device_step(bufs, segs, 77, step, advance=True, selected_count=cnt)
    refs = [h.copy() for h in hosts]
    ref_cnt = 0
    for replay in range(3):
        other = torch.from_numpy(hosts[0]).cuda()
        for k in range(18):
            wash.wash_shuffle(other, None, [(k + 3 + 50 * replay, 2000 + k, 0.2)], 0, 0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for r in refs:
            c = oracle.shuffle(r, None, segs_list, 77, 5 + replay)
        ref_cnt += c
        assert int(step.item()) == 6 + replay
        assert int(cnt.item()) == ref_cnt
        for b, r in zip(bufs, refs):
            assert np.array_equal(b.cpu().numpy().view(np.uint32), r.view(np.uint32)), replay
