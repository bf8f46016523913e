"""The streaming probe (fs_stream_probe) is what the benchmark's ceilings come from; its contract is checked here:
what it writes is the XOR of the streams it read and the element index, it touches nothing outside its streams, and a
read-only probe writes nothing."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("reads,writes", [(1, 1), (2, 1), (4, 1), (3, 2), (0, 1), (2, 0)])
@pytest.mark.parametrize("vecs", [1, 2, 4])
@pytest.mark.parametrize("n_vec,pad_vec", [(1, 0), (255, 0), (256 * 4 * 3 + 77, 0), (5000, 123)])
def test_probe_moves_exactly_its_streams(reads, writes, vecs, n_vec, pad_vec):
    import torch
    from paper_2009_10924_amd import binding as B
    rng = np.random.default_rng([reads, writes, vecs, n_vec])
    pitch_vec = n_vec + pad_vec
    guard = 64                                                   # vectors on each side that must stay as they are
    src_len = (max(reads, 1) - 1) * pitch_vec + n_vec
    dst_len = (max(writes, 1) - 1) * pitch_vec + n_vec
    src_host = rng.integers(0, 2 ** 32, size=(src_len, 4), dtype=np.uint32)
    dst_host = rng.integers(0, 2 ** 32, size=(dst_len + 2 * guard, 4), dtype=np.uint32)
    src = torch.from_numpy(src_host.view(np.int32)).cuda()
    dst = torch.from_numpy(dst_host.view(np.int32)).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    B.bind_probe(dst.data_ptr() + guard * 16, src.data_ptr(), n_vec * 16, reads, writes, vecs, stream, pitch_vec * 16)()
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint32)
    want = dst_host.copy()
    if writes:
        value = np.repeat(np.arange(n_vec, dtype=np.uint32)[:, None], 4, axis=1)
        for r in range(reads):
            value = value ^ src_host[r * pitch_vec:r * pitch_vec + n_vec]
        for w in range(writes):
            want[guard + w * pitch_vec:guard + w * pitch_vec + n_vec] = value
    assert np.array_equal(got, want)                              # the streams, and nothing before, between or behind them
