"""The measurement aids of wash_bench.h on the GPU: the copy copies, and the scattered-access probe stays
inside the buffer it is given (guard words on both sides keep their value) in every mode."""
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def wash():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2405_17517_amd as w
    return w


@pytest.mark.parametrize("n", [1, 5, 1024, 1027, 3 * 1024 * 1024 + 3])
def test_copy_copies(wash, n):
    print(f"case n={n}", flush=True)
    src = torch.randn(n, device="cuda:0")
    dst = torch.full((n + 8,), 7.0, device="cuda:0")
    wash.wash_copy_f32(src, dst[:n])
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src)
    assert bool((dst[n:] == 7.0).all())


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("lines", [2, 64, 1 << 14])
def test_probe_stays_inside_its_buffer(wash, mode, lines):
    print(f"case mode={mode} lines={lines}", flush=True)
    guard = 64                                         # words; keeps the inner buffer 256-byte aligned
    whole = torch.full((guard + lines * 32 + guard,), -3.0, device="cuda:0")
    inner = whole[guard:guard + lines * 32]
    mark = 0x7FC12345                                  # a bit pattern the probe is most unlikely to store
    inner.view(torch.int32).fill_(mark)
    places = wash.wash_probe_scattered(inner, mode, 2, 3)
    torch.cuda.synchronize()
    assert places == 3 * 256 * 2 * 8 // (4 if mode == 3 else 1)
    assert bool((whole[:guard] == -3.0).all()) and bool((whole[guard + lines * 32:] == -3.0).all())
    written = inner.view(torch.int32) != mark
    if mode == 0:
        assert int(written.sum()) == 0                 # loads only
    elif mode == 1:
        assert int(written.sum()) > 0
    elif mode == 3:
        # whole 64-byte pieces: a piece is written by four threads, 16 bytes each, or not at all
        per_piece = written.view(-1, 16).sum(dim=1)
        assert int(per_piece.sum()) > 0
        assert bool(((per_piece == 0) | (per_piece == 16)).all())
