"""The read-only measurement kernel (lutgemm_stream_read) really reads every byte once:
the XOR it leaves equals the XOR of the buffer, for sizes around its unrolling."""
import numpy as np
import pytest

import paper_2206_09557_amd as L
from gpu_util import torch_cuda

pytestmark = pytest.mark.gpu

SINK_WORDS = 8192
FULL = 2048 * 256 * 8      # 16-byte elements of one fully unrolled pass of every workgroup


@pytest.mark.parametrize("n16", [1, 63, 1024, 512 * 1024 + 7, FULL - 1, FULL, FULL + 1, 2 * FULL + 12345])
def test_xor_of_everything_read(n16):
    print(f"case n16={n16}", flush=True)
    torch = torch_cuda()
    rng = np.random.default_rng(6000 + n16 % 1000)
    host = rng.integers(0, 2**32, size=4 * n16, dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).cuda()
    sink = torch.full((SINK_WORDS,), -1, dtype=torch.int32, device="cuda")
    L.lutgemm_stream_read(src, 16 * n16, sink, 4 * SINK_WORDS, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host)


def test_rejects_bad_arguments():
    torch = torch_cuda()
    src = torch.zeros(64, dtype=torch.int32, device="cuda")
    sink = torch.zeros(SINK_WORDS, dtype=torch.int32, device="cuda")
    for args, code in [((src, 24, sink, 4 * SINK_WORDS), L.LUTGEMM_EINVAL),
                       ((src, 0, sink, 4 * SINK_WORDS), L.LUTGEMM_EINVAL),
                       ((src.data_ptr() + 4, 16, sink, 4 * SINK_WORDS), L.LUTGEMM_EINVAL),
                       ((src, 64, sink, 4 * SINK_WORDS - 4), L.LUTGEMM_EWORKSPACE)]:
        with pytest.raises(L.LutGemmError) as e:
            L.lutgemm_stream_read(*args)
        assert e.value.code == code
