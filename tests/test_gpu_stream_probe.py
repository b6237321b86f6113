"""cat_stream_probe: the measurement aid that only reads, or only copies, a buffer."""
import pytest
import torch

from paper_2509_26277_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 4096, 1 << 20, (1 << 24) + 48, 3 * 1000 * 1000 * 16])
def test_copy_mode_copies_every_byte_and_nothing_else(nbytes):
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    big = torch.full((nbytes + 512,), 7, dtype=torch.uint8, device="cuda")
    dst = big[256:256 + nbytes]
    binding.stream_probe(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert (big[:256] == 7).all() and (big[256 + nbytes:] == 7).all()
    binding.stream_probe(src)  # read only: nothing to check but that it runs and leaves src alone
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_bad_arguments_are_refused():
    src = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.CatError):
        binding.stream_probe(src[:24])          # not a multiple of 16
    with pytest.raises(binding.CatError):
        binding.stream_probe(src[8:40])         # misaligned
    with pytest.raises(ValueError):
        binding.stream_probe(src, src[:32])
