"""The two measurement aids of the library (plain copy, plain read) on the GPU."""
import pytest
import torch

from paper_2605_14305_amd import binding as fb

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def test_copy_probe_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    fb.fef_copy_probe(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_read_probe_reads_in_bounds_and_leaves_the_sink_alone():
    # a size that is no multiple of the grid's share (ragged last workgroup) and a tiny one
    for n in (1 << 22, (1 << 22) + 4 * 1237, 4):
        src = torch.full((n,), 3, dtype=torch.int32, device=DEV)
        sink = torch.zeros(1, dtype=torch.int32, device=DEV)
        fb.fef_read_probe(src, sink)
        torch.cuda.synchronize()
        assert int(sink.item()) == 0


def test_read_probe_reads_every_word_once():
    """The sink is written iff some thread's words XOR to one particular value: plant that value in one
    word of an otherwise zero buffer (inside the 128 KB blocks, at their edges, in the linear tail) and
    the sink must be set, which it is only if that word was read an odd number of times."""
    n = 5 * (1 << 15) * 7 + 4 * 1237          # 35 blocks of 128 KB and a tail of 4948 words
    magic = 0x9E3779B9 - (1 << 32)
    for pos in (0, 1, 12345, (1 << 15) - 1, 1 << 15, 17 * (1 << 15) + 511 * 4, 35 * (1 << 15) - 1, 35 * (1 << 15),
                n - 5, n - 1):
        src = torch.zeros(n, dtype=torch.int32, device=DEV)
        src[pos] = magic
        sink = torch.zeros(1, dtype=torch.int32, device=DEV)
        fb.fef_read_probe(src, sink)
        torch.cuda.synchronize()
        assert int(sink.item()) == 1, pos


def test_probes_reject_bad_arguments():
    src = torch.zeros(8, dtype=torch.int32, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(fb.FefError):
        fb.fef_read_probe(src[:3], sink)            # 12 bytes
    with pytest.raises(fb.FefError):
        fb.fef_read_probe(src[1:5], sink)           # misaligned
    with pytest.raises(fb.FefError):
        fb.fef_copy_probe(src[1:5], src[4:8])
