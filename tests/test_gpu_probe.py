"""The streaming-read yardstick (wkv_probe_read) really reads what it is asked to read.

The kernel has one observable effect: a lane whose loaded words XOR to a fixed constant writes that
constant to the sink.  A buffer of zeros with the constant planted in one word therefore sets the
sink exactly when the lane that owns that 16-byte piece has loaded it."""
import pytest
import torch

from paper_2503_01330_amd import binding as wkv

pytestmark = pytest.mark.gpu

MAGIC = 0x9E3779B9 - (1 << 32)          # as a signed 32-bit value


@pytest.mark.parametrize("nontemporal", [False, True])
@pytest.mark.parametrize("groups,threads,rounds", [(256, 1024, 3), (128, 512, 2), (7, 64, 5)])
def test_every_piece_of_the_buffer_is_loaded(groups, threads, rounds, nontemporal):
    dev = torch.device("cuda:0")
    per_group = 4 * threads * rounds                       # 16-byte pieces per workgroup: whole passes of 4 loads per lane
    words = groups * per_group * 4
    buf = torch.zeros(words, dtype=torch.int32, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def probe():
        wkv.wkv_probe_read(buf.data_ptr(), words * 4, groups, threads, nontemporal, sink.data_ptr(), stream)
        torch.cuda.synchronize()
        return int(sink.item())

    assert probe() == 0                                    # nothing planted: the sink is left alone
    g = torch.Generator().manual_seed(groups * 1000 + threads)
    spots = [0, words - 1, per_group * 4 - 1, per_group * 4] + torch.randint(0, words, (12,), generator=g).tolist()
    for w in spots:
        buf[w] = MAGIC
        assert probe() == MAGIC, f"word {w} of {words} was not read"
        buf[w] = 0
        sink.zero_()
    assert probe() == 0


def test_argument_checks():
    dev = torch.device("cuda:0")
    buf = torch.zeros(1 << 16, dtype=torch.int32, device=dev)
    ok = dict(workgroups=16, threads=256, nontemporal=False)
    with pytest.raises(wkv.WkvError):
        wkv.wkv_probe_read(0, 1 << 18, **ok)
    with pytest.raises(wkv.WkvError):
        wkv.wkv_probe_read(buf.data_ptr() + 4, 1 << 17, **ok)              # not 16-byte aligned
    with pytest.raises(wkv.WkvError):
        wkv.wkv_probe_read(buf.data_ptr(), (1 << 17) + 16, **ok)           # not a multiple of 16 * workgroups
    with pytest.raises(wkv.WkvError):
        wkv.wkv_probe_read(buf.data_ptr(), 1 << 17, workgroups=16, threads=100, nontemporal=False)
    wkv.wkv_probe_read(buf.data_ptr(), 1 << 18, **ok)
    torch.cuda.synchronize()
