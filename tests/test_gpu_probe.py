"""wgkv_stream_read_probe, the plain streaming read bench.py times as the live ceiling of the machine: it must read
every 16-byte piece of the range it is given and write nothing but its sink.  A lane XORs the words it reads and
stores to the sink only if the result is one particular constant, so a buffer of zeros with that constant in one
word shows whether the piece holding the word was read."""
import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from paper_2512_17452_amd.binding import stream_read_probe

pytestmark = pytest.mark.gpu

MAGIC = 0x9E3779B9


@pytest.mark.parametrize("n_bytes", [16, 4096, 1 << 20, (1 << 22) + 16 * 12345, (256 * 256 * 8 * 16) * 3 + 16 * 7])
def test_probe_reads_every_piece_and_writes_only_its_sink(n_bytes):
    dev = torch.device("cuda:0")
    buf = torch.zeros(n_bytes + 64, dtype=torch.uint8, device=dev)
    words = buf[:n_bytes].view(torch.int32)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    rng = np.random.default_rng(n_bytes)
    n_words = n_bytes // 4
    places = sorted({0, n_words - 1, n_words - 4, n_words // 2} | {int(x) for x in rng.integers(0, n_words, 5)})
    for w in places:
        words.zero_()
        sink.zero_()
        words[w] = np.int32(np.uint32(MAGIC).astype(np.int32))
        before = buf.clone()
        stream_read_probe(buf, n_bytes, sink)
        torch.cuda.synchronize()
        assert int(sink[0].item()) & 0xFFFFFFFF == MAGIC, f"word {w} of {n_words} was not read"
        assert torch.equal(buf, before) and int(sink[1:].abs().sum().item()) == 0
    # a word past the range is not part of it
    words.zero_()
    sink.zero_()
    buf[n_bytes:n_bytes + 4].view(torch.int32)[0] = np.int32(np.uint32(MAGIC).astype(np.int32))
    stream_read_probe(buf, n_bytes, sink)
    torch.cuda.synchronize()
    assert int(sink[0].item()) == 0


def test_probe_refuses_bad_arguments():
    dev = torch.device("cuda:0")
    buf = torch.zeros(4096, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for args in [(buf, 8, sink), (buf[4:], 1024, sink)]:
        with pytest.raises(wg.WgkvError) as e:
            stream_read_probe(*args)
        assert e.value.code == -1
