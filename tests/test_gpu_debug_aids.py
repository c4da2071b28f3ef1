"""GPU checks of the measurement aids (bitsnap_debug_stream_copy, bitsnap_debug_stream_mix): the copy
kernel calibrates the HBM byte counters, so it has to move exactly what it says; the byte-mix kernels only
have to stay inside their buffers and touch all of them."""
import pytest
import torch

from gpu_util import DEV, announce
from paper_2511_12376_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 48, 16 * 1023, 16 * 1024, 16 * 1025, 16 * 4096 + 32, 3 * (1 << 20) + 16 * 777, 320_864_256])
def test_stream_copy_moves_every_byte_and_nothing_else(nbytes):
    announce("debug stream copy", nbytes)
    g = torch.Generator(device=DEV)
    g.manual_seed(nbytes)
    pad = 4096
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g)
    buf = torch.full((nbytes + 2 * pad,), 0xA5, dtype=torch.uint8, device=DEV)
    dst = buf[pad:pad + nbytes]
    B.debug_stream_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert bool((buf[:pad] == 0xA5).all()) and bool((buf[pad + nbytes:] == 0xA5).all())


@pytest.mark.parametrize("groups", [1, 3, 15, 16, 17, 1000])
def test_stream_mix_stays_inside_its_buffers(groups):
    announce("debug stream mix", groups)
    n, pad = groups * 4096, 4096
    wide_buf = torch.full((n + 2 * pad,), 7.0, dtype=torch.float32, device=DEV)
    bytes_buf = torch.full((n + 2 * pad,), 0x5A, dtype=torch.uint8, device=DEV)
    halves_buf = torch.full((n // 2 + 2 * pad,), 0x5A, dtype=torch.uint8, device=DEV)
    wide, small, halves = wide_buf[pad:pad + n], bytes_buf[pad:pad + n], halves_buf[pad:pad + n // 2]
    wide.copy_(torch.arange(n, device=DEV, dtype=torch.float32))
    B.debug_stream_mix(wide, small, halves, True)    # wide -> small, halves
    torch.cuda.synchronize()
    assert bool((wide_buf[:pad] == 7.0).all()) and bool((wide_buf[pad + n:] == 7.0).all())
    for buf, m in ((bytes_buf, n), (halves_buf, n // 2)):
        assert bool((buf[:pad] == 0x5A).all()) and bool((buf[pad + m:] == 0x5A).all())
    wide.fill_(-1.0)
    B.debug_stream_mix(wide, small, halves, False)   # small, halves -> wide
    torch.cuda.synchronize()
    assert bool((wide >= 0.0).all())                 # every element was written (bytes turned into numbers are >= 0)
    assert bool((wide_buf[:pad] == 7.0).all()) and bool((wide_buf[pad + n:] == 7.0).all())
