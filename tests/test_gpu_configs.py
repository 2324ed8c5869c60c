"""GPU parity at the full sizes of the five benchmark configurations, in the
launch configuration bench.py times (default tile choice, count requested).

All five configs are compared element by element over the whole population:
configs 1-4 against an oracle copy on the host, config 5 (70 GB with momentum)
chunk by chunk against a device copy of its initial state (the stream is
addressed by the global coordinate, so the oracle can shuffle a window on its
own)."""
import math
import os

import numpy as np
import pytest

import oracle
from workloads import device_population, get_config

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

THREADS = max(1, min(16, os.cpu_count() or 1))


@pytest.fixture(scope="module")
def wash():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_17517_amd as w
    w.wash_set_option(w.OPT_TILE_COORDS, 0)
    return w


def _bits(a):
    return a.view(np.uint32)


def _close(got, ref, pop_abs_mean):
    scale = np.maximum(np.abs(ref), pop_abs_mean)
    return bool(np.all(np.abs(got - ref) <= 1e-6 * scale))


def _full_config(wash, index, steps, p_values=(None,), check_ema=True, stream="v1"):
    shuffle = wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap
    cfg = get_config(index)
    pop, mom = device_population(cfg.tensors(), cfg.N, cfg.init, cfg.data_seed, cfg.momentum)
    ref = pop.cpu().numpy()
    refm = mom.cpu().numpy() if mom is not None else None
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    ref_cnt, step = 0, 0
    for p in p_values:
        segs_list = cfg.segments(p)
        segs = wash.SegmentList(segs_list)
        for _ in range(steps):
            print(f"config {index} p={p} step {step} stream {stream}", flush=True)
            shuffle(pop, mom, segs, cfg.seed, step, cnt)
            ref_cnt += oracle.shuffle(ref, refm, segs_list, cfg.seed, step, threads=THREADS, stream=stream)
            step += 1
    torch.cuda.synchronize()
    assert int(cnt.item()) == ref_cnt and ref_cnt > 0
    got = pop.cpu().numpy()
    assert np.array_equal(_bits(got), _bits(ref)), "params differ from the oracle"
    del got
    if mom is not None:
        assert np.array_equal(_bits(mom.cpu().numpy()), _bits(refm)), "momentum differs from the oracle"
    abs_mean = np.abs(ref).mean(axis=0)
    avg = wash.wash_average(pop).cpu().numpy()
    ref_avg = oracle.average(ref)
    assert _close(avg, ref_avg, abs_mean), "average outside 1e-6"
    if check_ema:
        wash.papa_ema(pop, cfg.alpha)
        oracle.ema(ref, cfg.alpha)
        assert _close(pop.cpu().numpy(), ref, abs_mean[None, :]), "EMA outside 1e-6"


STREAMS = ["v1", "gap"]


@pytest.mark.parametrize("stream", STREAMS)
def test_config1_flat(wash, stream):
    _full_config(wash, 1, steps=1, stream=stream)


@pytest.mark.parametrize("stream", STREAMS)
def test_config2_resnet18_100_steps(wash, stream):
    _full_config(wash, 2, steps=100, stream=stream, check_ema=(stream == "v1"))


@pytest.mark.parametrize("stream", STREAMS)
def test_config3_resnet50_momentum_100_steps(wash, stream):
    _full_config(wash, 3, steps=100, stream=stream, check_ema=(stream == "v1"))


@pytest.mark.parametrize("stream", STREAMS)
def test_config4_vit_p_sweep(wash, stream):
    cfg = get_config(4)
    _full_config(wash, 4, steps=2, p_values=cfg.p_sweep, stream=stream, check_ema=(stream == "v1"))


@pytest.mark.parametrize("stream", STREAMS)
def test_config5_whole_population(wash, stream):
    """Config 5 (N = 8, P = 1.1e9, params + momentum, 10 steps, then average and EMA) compared with the
    oracle on EVERY coordinate.  The 70 GB population cannot sit beside an oracle copy on the host, so a
    device copy of the initial state is kept (5 x 35 GB on the device in all) and the row is walked in
    chunks of 2^20 columns: initial and final chunks are downloaded, the oracle replays all steps on the
    initial chunk (its stream is addressed by the global coordinate), and parameters, momentum, the
    average and the EMA of the chunk are compared; the selected count must equal the oracle's."""
    from concurrent.futures import ThreadPoolExecutor

    shuffle = wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap
    cfg = get_config(5)
    N, P, steps, alpha = cfg.N, cfg.P, cfg.steps, cfg.alpha
    segs_list = cfg.segments()
    segs = wash.SegmentList(segs_list)
    pop, mom = device_population(cfg.tensors(), N, cfg.init, cfg.data_seed, True)
    pop0, mom0 = pop.clone(), mom.clone()
    print(f"config 5 generated, stream {stream}", flush=True)

    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    for step in range(steps):
        shuffle(pop, mom, segs, cfg.seed, step, cnt)
    avg = wash.wash_average(pop)
    ema = pop.clone()
    wash.papa_ema(ema, alpha)
    torch.cuda.synchronize()
    print("config 5 shuffled, averaged, EMA applied", flush=True)

    W = 1 << 20

    def check(g0, blk, avg_chunk):
        """blk: host [5, N, w] = initial params, initial momentum, final params, final momentum, EMA."""
        w = blk.shape[2]
        ref, refm = blk[0], blk[1]
        local = [sg for sg in segs_list if sg[0] < g0 + w and sg[0] + sg[1] > g0]
        c = 0
        for step in range(steps):
            c += oracle.shuffle_window(ref, refm, P, g0, local, cfg.seed, step, stream=stream)
        assert np.array_equal(_bits(blk[2]), _bits(ref)), f"params differ in the chunk at {g0}"
        assert np.array_equal(_bits(blk[3]), _bits(refm)), f"momentum differs in the chunk at {g0}"
        abs_mean = np.abs(ref).mean(axis=0)
        assert _close(avg_chunk, oracle.average(ref), abs_mean), f"average outside 1e-6 in the chunk at {g0}"
        oracle.ema(ref, alpha)
        assert _close(blk[4], ref, abs_mean[None, :]), f"EMA outside 1e-6 in the chunk at {g0}"
        return c

    ref_cnt, pending, done = 0, [], 0
    with ThreadPoolExecutor(max_workers=THREADS) as pool:
        for g0 in range(0, P, W):
            g1 = min(P, g0 + W)
            blk = torch.stack([t[:, g0:g1] for t in (pop0, mom0, pop, mom, ema)]).cpu().numpy()
            pending.append(pool.submit(check, g0, blk, avg[g0:g1].cpu().numpy()))
            while len(pending) > 2 * THREADS:
                ref_cnt += pending.pop(0).result()
                done += 1
                if done % 128 == 0:
                    print(f"config 5: {done} chunks compared", flush=True)
        for f in pending:
            ref_cnt += f.result()
    assert int(cnt.item()) == ref_cnt and ref_cnt > 0
    # Table 1's volume: the count is what Sec. 3 calls the communication per model, sum_s p_s * len_s per step
    mean = steps * sum(length * p for _, length, p in segs_list)
    var = steps * sum(length * p * (1 - p) for _, length, p in segs_list)
    assert abs(ref_cnt - mean) < 6 * math.sqrt(var)


@pytest.mark.parametrize("nbuf", [3, 4])
def test_dense_path_beyond_4gib_with_several_states(wash, nbuf):
    """WASH+Opt with 3 and 4 buffers at p = 0.1 on more than 4 GiB: the streaming (dense) kernel with
    non-temporal accesses, which smaller cases never reach.  Every buffer must end up as the oracle
    leaves it when it shuffles that buffer alone with the same (seed, step)."""
    N, P = 8, 46_000_003
    assert N * P * 4 * nbuf >= 4 << 30
    segs_list = [(0, P // 3, 0.1), (P // 3, P - P // 3 - 5, 0.25), (P - 5, 5, 1.0)]
    gen = torch.Generator(device="cuda").manual_seed(41 + nbuf)
    bufs = [torch.randn(N, P, device="cuda", generator=gen) * (0.02 if k == 0 else 1e-3) for k in range(nbuf)]
    hosts = [b.cpu().numpy() for b in bufs]
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    print(f"dense path, {nbuf} buffers, {N * P * 4 * nbuf / 2**30:.1f} GiB", flush=True)
    wash.wash_shuffle_states(bufs, segs_list, 17, 3, gap_stream=False, selected_count=cnt)
    torch.cuda.synchronize()
    for k, (b, h) in enumerate(zip(bufs, hosts)):
        ref_cnt = oracle.shuffle(h, None, segs_list, 17, 3, threads=THREADS)
        assert int(cnt.item()) == ref_cnt
        assert np.array_equal(_bits(b.cpu().numpy()), _bits(h)), f"buffer {k} differs from the oracle"


@pytest.mark.parametrize("stream", STREAMS)
def test_coordinates_beyond_two_to_the_32(wash, stream):
    """Rows longer than 2^32 coordinates: the high words of the coordinate enter the Philox counters
    (permutation words from g = 2^32 on, mask quads through g >> 2).  N = 2 with momentum, 69 GB on
    the device; compared with the oracle on windows around the 2^32 mark, at both ends, and through
    the per-coordinate fingerprints over the whole rows."""
    shuffle = wash.wash_shuffle if stream == "v1" else wash.wash_shuffle_gap
    N, two32 = 2, 1 << 32
    P = two32 + (1 << 21) + 5
    segs_list = [(0, two32 - 1000, 0.0005), (two32 - 1000, 2000 + (1 << 20), 0.5)]
    rest = segs_list[-1][0] + segs_list[-1][1]
    segs_list.append((rest, P - rest, 0.01))
    segs = wash.SegmentList(segs_list)

    def generate(salt):
        t = torch.empty(N, P, dtype=torch.float32, device="cuda")
        v = t.view(torch.int32)
        chunk = 1 << 28
        for n in range(N):
            for c0 in range(0, P, chunk):
                c1 = min(P, c0 + chunk)
                idx = torch.arange(c0, c1, device="cuda", dtype=torch.int64)
                # any 32-bit patterns will do (values are moved bit for bit); keep them finite floats
                v[n, c0:c1] = (((idx * 0x9E3779 + (n + salt) * 0x85EBCA6B) >> 5) & 0x3FFFFFFF).to(torch.int32)
        return t

    pop, mom = generate(1), generate(11)
    print("long rows generated", flush=True)

    def fold(t):
        v = t.view(torch.int32)
        return v[0] ^ v[1], v[0] + v[1]

    fx, fs = fold(pop)
    mx, ms = fold(mom)
    W = 1 << 20
    starts = [0, two32 - W // 2, two32 + (1 << 20) - 4096, (P - W) // 1024 * 1024, (1 << 31) - 2048, 3 * (1 << 30)]
    widths = [W if g0 + W + 1024 < P else P - g0 for g0 in starts]
    init = [(pop[:, g0:g0 + w].clone(), mom[:, g0:g0 + w].clone()) for g0, w in zip(starts, widths)]

    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    tiles = [0, 512] if stream == "v1" else [0, 0]
    for step, tile in enumerate(tiles):
        wash.wash_set_option(wash.OPT_TILE_COORDS, tile)
        shuffle(pop, mom, segs, 0xABCDEF0123456789, step, cnt)
    wash.wash_set_option(wash.OPT_TILE_COORDS, 0)
    torch.cuda.synchronize()
    print("long rows shuffled", flush=True)

    gx, gs = fold(pop)
    assert torch.equal(gx, fx) and torch.equal(gs, fs)
    del fx, fs, gx, gs
    gx, gs = fold(mom)
    assert torch.equal(gx, mx) and torch.equal(gs, ms)
    del mx, ms, gx, gs
    steps = len(tiles)
    mean = steps * sum(length * p for _, length, p in segs_list)
    var = steps * sum(length * p * (1 - p) for _, length, p in segs_list)
    assert abs(int(cnt.item()) - mean) < 6 * math.sqrt(var)

    avg = wash.wash_average(pop)
    refs = []
    for g0, w, (ip, im) in zip(starts, widths, init):
        print(f"long rows window at {g0} width {w}", flush=True)
        ref, refm = ip.cpu().numpy(), im.cpu().numpy()
        for step in range(steps):
            oracle.shuffle_window(ref, refm, P, g0, segs_list, 0xABCDEF0123456789, step, stream=stream)
        assert np.array_equal(_bits(pop[:, g0:g0 + w].contiguous().cpu().numpy()), _bits(ref)), f"params window {g0}"
        assert np.array_equal(_bits(mom[:, g0:g0 + w].contiguous().cpu().numpy()), _bits(refm)), f"momentum window {g0}"
        assert not np.array_equal(_bits(ref), _bits(ip.cpu().numpy()))
        assert _close(avg[g0:g0 + w].cpu().numpy(), oracle.average(ref), np.abs(ref).mean(axis=0)), f"average {g0}"
        refs.append(ref)
    # the streaming kernels index rows of more than 2^32 elements as well
    wash.papa_ema(pop, 0.75)
    for g0, w, ref in zip(starts, widths, refs):
        abs_mean = np.abs(ref).mean(axis=0)
        oracle.ema(ref, 0.75)
        assert _close(pop[:, g0:g0 + w].contiguous().cpu().numpy(), ref, abs_mean[None, :]), f"EMA window {g0}"


@pytest.mark.parametrize("base_p", [0.5, 1.0])
def test_layerwise_schedule_with_a_large_base_probability(wash, base_p):
    """Eq. 6 on the ResNet-18 tensor list with the base probabilities of the paper's ablation: the
    first tensors are dense enough for the streaming path, the last ones are not, so one call runs
    both kernels on their parts of the list.  Two steps, momentum moved along, whole population
    compared with the oracle."""
    from workloads import layouts
    cfg = get_config(2)
    tensors = cfg.tensors()
    probs = wash.wash_layer_probs(base_p, len(tensors), 0)
    assert probs[0] == base_p and probs[-1] == 0.0 and min(probs[:-1]) > 0.0
    segs_list = layouts.segments_of(tensors, probs)
    segs = wash.SegmentList(segs_list)
    pop, _ = device_population(tensors, cfg.N, cfg.init, cfg.data_seed, False)
    mom = torch.randn(cfg.N, cfg.P, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)) * 1e-3
    ref, refm = pop.cpu().numpy(), mom.cpu().numpy()
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    ref_cnt = 0
    for step in range(2):
        print(f"layer-wise schedule base {base_p} step {step}", flush=True)
        wash.wash_shuffle(pop, mom, segs, 11, step, cnt)
        ref_cnt += oracle.shuffle(ref, refm, segs_list, 11, step, threads=THREADS)
    torch.cuda.synchronize()
    assert int(cnt.item()) == ref_cnt
    # Table 1's volume: half of base_p * d per step when every layer has the same size; here weighted by size
    expect = 2 * sum(length * p for _, length, p in segs_list)
    assert abs(ref_cnt - expect) < 6 * math.sqrt(expect)
    assert np.array_equal(_bits(pop.cpu().numpy()), _bits(ref))
    assert np.array_equal(_bits(mom.cpu().numpy()), _bits(refm))
