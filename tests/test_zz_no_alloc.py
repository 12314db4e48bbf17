"""The entry point that allocates nothing: quest_lowbit_gemm_static (built-in scratch buffer) against
quest_lowbit_gemm with a caller workspace, bit for bit, on two calls in a row, the second smaller.

Collected last (file name): the buffer it uses is shared by every call on the GPU."""
import numpy as np
import pytest
import torch

from paper_2502_05003_amd import binding as q

from gpu_util import DEV, lowbit_ws

pytestmark = pytest.mark.gpu


def _operands(M, N, K, bits, seed):
    """Random packed codes (every code value, bytes drawn uniformly) and positive scales."""
    rng = np.random.default_rng(seed)
    cb = q.quest_container_bits(bits)
    a = torch.from_numpy(rng.integers(0, 256, size=(M, K * cb // 8), dtype=np.uint8)).to(DEV)
    b = torch.from_numpy(rng.integers(0, 256, size=(N, K * cb // 8), dtype=np.uint8)).to(DEV)
    sa = torch.from_numpy((rng.random(M) + 0.5).astype(np.float32)).to(DEV)
    sb = torch.from_numpy(((rng.random(N) + 0.5) * 0.01).astype(np.float32)).to(DEV)
    return a, sa, b, sb


@pytest.mark.parametrize("bits", [2, 1])
def test_static_scratch_entry_point_matches_the_workspace_one(bits):
    # first call: 14 MiB of scratch, ragged tiles; second call: a smaller shape over the same buffer
    for seed, (M, N, K) in enumerate([(9000, 5000, 2048), (700, 600, 512)]):
        a, sa, b, sb = _operands(M, N, K, bits, seed)
        assert 0 < q.quest_lowbit_gemm_workspace_bytes(M, N, K, bits) <= 32 << 20
        y_ref = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
        acc_ref = torch.empty(M, N, dtype=torch.int32, device=DEV)
        q.quest_lowbit_gemm(a, sa, b, sb, K, bits, y=y_ref, acc_out=acc_ref, workspace=lowbit_ws(M, N, K, bits))
        y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
        q.quest_lowbit_gemm_static(a, sa, b, sb, K, bits, y=y, acc_out=acc)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc_ref), (bits, M, N, K)
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (bits, M, N, K)
        assert int(acc_ref.abs().max()) > 0


def test_static_entry_point_rejects_what_its_buffer_cannot_hold():
    M, N, K = 65536, 8192, 1024      # (M + N) K / 2 = 36 MiB > 32 MiB
    a = torch.zeros(16, dtype=torch.uint8, device=DEV)       # never read: the size check comes first
    s = torch.zeros(16, dtype=torch.float32, device=DEV)
    lib = q.load()
    status = lib.quest_lowbit_gemm_static(a.data_ptr(), s.data_ptr(), M, a.data_ptr(), s.data_ptr(), N, K, 2,
                                          a.data_ptr(), N, None, None)
    assert status == 9
