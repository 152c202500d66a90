"""GPU check of the streaming-read calibration kernel (measurement support)."""
import numpy as np
import pytest

from paper_2311_18677_amd import binding as sw

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_words,wg", [(4, 1), (4 * 1000, 3), (4 * 70001, 0), (4 * 2048 * 256 * 9 + 4 * 77, 2048), (0, 5)])
def test_stream_read_xor_of_all_words(n_words, wg):
    import torch
    rng = np.random.Generator(np.random.Philox(900 + n_words % 1000))
    host = rng.integers(0, 2 ** 32, size=max(n_words, 4), dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).to("cuda:0")
    groups = wg if wg else 16384          # room for the library's own choice
    sink = torch.full((groups,), -1, dtype=torch.int32, device="cuda:0")
    print("stream read", n_words, wg, flush=True)
    sw.sw_stream_read(src, 4 * n_words, sink, wg)
    torch.cuda.synchronize()
    words = sink.cpu().numpy().view(np.uint32)
    if not wg:
        words = words[words != np.uint32(0xFFFFFFFF)]      # entries past the library's grid keep the fill
    got = np.bitwise_xor.reduce(words) if words.size else np.uint32(0)
    want = np.bitwise_xor.reduce(host[:n_words]) if n_words else np.uint32(0)
    assert got == want
