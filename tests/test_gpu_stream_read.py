"""The streaming-read reference kernel reads every 16-byte group exactly once: the sum of its
per-workgroup checksums equals the sum, over all groups, of the XOR of the group's four words."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n16", [1, 255, 256, 257, 8 * 8192 * 256 - 1, 8 * 8192 * 256 + 12345, 2 * 8 * 8192 * 256 + 1])
def test_stream_read_touches_every_group_once(n16):
    import torch
    import paper_2401_18079_amd as K
    rng = np.random.default_rng(n16)
    words = rng.integers(0, 2**32, size=(n16, 4), dtype=np.uint64).astype(np.uint32)
    buf = torch.from_numpy(words.view(np.int32)).cuda()
    ws = torch.zeros(K.binding.kvq_stream_read_workspace_bytes() // 4, dtype=torch.int32, device="cuda")
    K.kvq_stream_read(buf, ws)
    got = int(ws.cpu().numpy().view(np.uint32).astype(np.uint64).sum() % 2**32)
    x = words[:, 0] ^ words[:, 1] ^ words[:, 2] ^ words[:, 3]
    assert got == int(x.astype(np.uint64).sum() % 2**32)


def test_stream_read_argument_errors():
    import torch
    import paper_2401_18079_amd as K
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(K.binding.kvq_stream_read_workspace_bytes(), dtype=torch.uint8, device="cuda")
    with pytest.raises(K.KvqError):
        K.kvq_stream_read(buf[:24], ws)                    # not a multiple of 16 bytes
    with pytest.raises(K.KvqError):
        K.kvq_stream_read(buf[4:36], ws)                   # not 16-byte aligned
    with pytest.raises(K.KvqError):
        K.kvq_stream_read(buf, ws[:64])                    # workspace too small
