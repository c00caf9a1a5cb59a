"""kunlun_stream_probe: the calibration kernel moves the bytes it is priced for, and nothing else."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import binding
    assert torch.cuda.is_available()
    return binding


@pytest.mark.parametrize("nbytes", [4096, 16 * 1024, 16 * 1025, (1 << 20) + 48])
@pytest.mark.parametrize("reads", [1, 2, 3])
def test_written_stream_is_the_xor_of_the_read_streams(kb, nbytes, reads):
    g = torch.Generator(device="cuda")
    g.manual_seed(nbytes + reads)
    a, b, c = (torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g) for _ in range(3))
    guard = 64
    out = torch.full((nbytes + guard,), 0xAB, dtype=torch.uint8, device="cuda")
    kb.stream_probe(a, b if reads > 1 else None, c if reads > 2 else None, out[:nbytes], reads, 1)
    want = a.clone()
    if reads > 1:
        want ^= b
    if reads > 2:
        want ^= c
    assert torch.equal(out[:nbytes], want)
    assert bool((out[nbytes:] == 0xAB).all()), "wrote past the end"


def test_read_only_pass_writes_nothing(kb):
    n = 1 << 20
    a = torch.ones(n, dtype=torch.uint8, device="cuda")
    out = torch.full((4096,), 0x5C, dtype=torch.uint8, device="cuda")
    kb.stream_probe(a, a, a, out, 3, 0)
    assert bool((out == 0x5C).all())


def test_rejects_bad_arguments(kb):
    a = torch.ones(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(kb.KunlunError):
        kb.stream_probe(a, None, None, a.clone(), 2, 1)      # second stream missing
    with pytest.raises(kb.KunlunError):
        kb.stream_probe(a, None, None, a.clone(), 4, 1)
    with pytest.raises(kb.KunlunError):
        kb.stream_probe(a[:4088], None, None, a.clone()[:4088], 1, 1)   # not a multiple of 16
