"""GPU test of cce_forward_static, the entry point that allocates nothing (its scratch is a static
device array inside the library), against cce_forward: same kernels and plan, so the outputs must be
the same bits.  Two calls in a row, the second with a smaller input: whatever the first call left in
the shared array must not leak into the second.  Collected last (file name) because a failure here
must not hide the other GPU tests behind pytest -x."""
import numpy as np
import pytest
import torch

from paper_2601_02609_amd import inputs as I
from tests.gpu_util import dev_inputs

pytestmark = pytest.mark.gpu
IGN = -100


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


def _both(B, w):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    ref_loss, ref_lse = B.cce_forward(H, W, y, IGN)
    loss = torch.full((N,), 7.0, device="cuda")
    lse = torch.full((N,), 7.0, device="cuda")
    status = torch.full((1,), 99, dtype=torch.int32, device="cuda")
    L = B.lib()
    rc = L.cce_forward_static(H.data_ptr(), W.data_ptr(), y.data_ptr(), N, D, V, IGN,
                              loss.data_ptr(), lse.data_ptr(), status.data_ptr(),
                              torch.cuda.current_stream().cuda_stream)
    assert rc == B.CCE_OK, L.cce_strerror(rc)
    torch.cuda.synchronize()
    return ref_loss, ref_lse, loss, lse, int(status.item())


def test_static_forward_equals_workspace_forward_twice_in_a_row(B):
    big = I.make_workload(I.custom_spec(1300, 256, 5000, seed=61, ignore_frac=0.2))
    small = I.make_workload(I.custom_spec(300, 128, 777, seed=62, ignore_frac=0.1))
    for tag, w in (("first call", big), ("second call, smaller input", small)):
        print(f"[static] {tag}: N={w.spec.N} D={w.spec.D} V={w.spec.V}", flush=True)
        ref_loss, ref_lse, loss, lse, status = _both(B, w)
        assert status == 0
        assert torch.equal(loss, ref_loss) and torch.equal(lse, ref_lse)
        ign = torch.from_numpy(w.labels == IGN).cuda()
        assert bool((loss[ign] == 0).all()) and bool((lse[ign] == 0).all())


def test_static_forward_status_and_limits(B):
    w = I.make_workload(I.custom_spec(100, 64, 300, seed=63, ignore_frac=0.0))
    w.labels[5] = 300                                   # out of range: flagged in the caller's status word
    ref_loss, ref_lse, loss, lse, status = _both(B, w)
    assert status & B.CCE_STATUS_BAD_LABEL and torch.equal(loss, ref_loss) and float(loss[5]) == 0.0
    # a clean call afterwards clears the word again
    w2 = I.make_workload(I.custom_spec(100, 64, 300, seed=64, ignore_frac=0.0))
    assert _both(B, w2)[4] == 0
    # beyond the static array: refused with its own error code, nothing launched
    L = B.lib()
    H, W, y = dev_inputs(w2)
    rc = L.cce_forward_static(H.data_ptr(), W.data_ptr(), y.data_ptr(), 1 << 22, 64, 300, IGN,
                              loss.data_ptr(), lse.data_ptr(), None, torch.cuda.current_stream().cuda_stream)
    assert rc == B.CCE_ERR_TOO_LARGE
    rc = L.cce_forward_static(None, W.data_ptr(), y.data_ptr(), 100, 64, 300, IGN,
                              loss.data_ptr(), lse.data_ptr(), None, torch.cuda.current_stream().cuda_stream)
    assert rc == B.CCE_ERR_INVALID
