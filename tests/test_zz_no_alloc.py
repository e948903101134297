"""The entry point that allocates nothing: po_op_colsum_accumulate_static against po_op_colsum_accumulate
(the same kernels with a caller workspace) and against the plain definition, two calls in a row on one
device, the second with a smaller input, so that whatever the first call left in the built-in scratch
array would show if the second one read it."""
import numpy as np
import pytest
import torch

from paper_2503_01328_amd import binding as po
from paper_2503_01328_amd import inputs as syn

pytestmark = pytest.mark.gpu


def _case(dev, dtype, rows, n, seed):
    code, tdt = (po.PO_BF16, torch.bfloat16) if dtype == "bf16" else (po.PO_F32, torch.float32)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, n), dtype=np.float32)
    if dtype == "bf16":
        x = syn.round_to_bf16(x)
    acc0 = rng.standard_normal(n, dtype=np.float32)
    xd = torch.from_numpy(x).to(dev).to(tdt).contiguous()
    ref_acc = torch.from_numpy(acc0.copy()).to(dev)
    ws = torch.empty(po.po_op_colsum_workspace(rows, n) // 4, dtype=torch.float32, device=dev)
    po.po_op_colsum_accumulate(code, xd, ref_acc, ws, rows, n)
    got_acc = torch.from_numpy(acc0.copy()).to(dev)
    before = torch.cuda.memory_allocated(dev)
    po.po_op_colsum_accumulate_static(code, xd, got_acc, rows, n)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(dev) == before
    assert torch.equal(got_acc, ref_acc), (dtype, rows, n)  # same kernels, same order: bit for bit
    want = acc0.astype(np.float64) + x.astype(np.float64).sum(0)
    err = np.abs(got_acc.cpu().numpy() - want).max() / np.abs(want).max()
    assert err < 1e-4, err  # fp32 sums of the given values in either dtype


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_colsum_two_calls_second_smaller(gpu_device, dtype):
    _case(gpu_device, dtype, 2048, 8192, 1)  # 64 row chunks x 8192 columns of partials
    _case(gpu_device, dtype, 100, 130, 2)    # 4 chunks x 130 columns: reads only what it wrote itself
    _case(gpu_device, dtype, 1, 2, 3)


def test_static_colsum_rejects_sizes_beyond_the_scratch(gpu_device):
    x = torch.zeros(4, 32770, dtype=torch.float32, device=gpu_device)
    acc = torch.zeros(32770, dtype=torch.float32, device=gpu_device)
    with pytest.raises(po.PipeOffloadError, match="32768"):
        po.po_op_colsum_accumulate_static(po.PO_F32, x, acc, 4, 32770)
    with pytest.raises(po.PipeOffloadError):
        po.po_op_colsum_accumulate_static(po.PO_F32, x, acc, 4, 3)  # odd n
    assert torch.count_nonzero(acc).item() == 0
