"""The compute calls are plain kernel launches on the caller's stream: they work on a
non-default stream and under HIP graph capture (replayed several times, with eager work and
synchronisation between the replays, each replay checked against the eager result)."""
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


def _buffers(B, w):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    return dict(H=H, W=W, y=y, dl=torch.from_numpy(w.dloss_mean).cuda(), ws=B.alloc_workspace(N, D, V),
                loss=torch.empty(N, device="cuda"), lse=torch.empty(N, device="cuda"),
                dH=torch.empty(N, D, dtype=torch.bfloat16, device="cuda"), dW=torch.empty(V, D, device="cuda"))


def _step(B, b, stream=None):
    B.cce_forward(b["H"], b["W"], b["y"], IGN, workspace=b["ws"], loss=b["loss"], lse=b["lse"], stream=stream)
    B.cce_backward(b["H"], b["W"], b["y"], b["lse"], b["dl"], IGN, workspace=b["ws"], d_hidden=b["dH"],
                   d_weight=b["dW"], stream=stream)


def test_non_default_stream_matches_default(B):
    w = I.make_workload(I.custom_spec(700, 896, 3000, seed=41, ignore_frac=0.2))
    a, b = _buffers(B, w), _buffers(B, w)
    _step(B, a)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        _step(B, b, stream=s)
    s.synchronize()
    for k in ("loss", "lse", "dH", "dW"):
        assert torch.equal(a[k], b[k]), k


def test_graph_capture_and_replay(B):
    w = I.make_workload(I.custom_spec(520, 128, 2100, seed=42, ignore_frac=0.1))
    ref, b = _buffers(B, w), _buffers(B, w)
    _step(B, ref)
    _step(B, b)                      # warm-up outside the capture (first-use set-up of the library)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            _step(B, b, stream=s)
    for rep in range(3):
        for k in ("loss", "lse", "dH", "dW"):
            b[k].zero_()
        junk = torch.randn(1 << 20, device="cuda").sum()      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ("loss", "lse", "dH", "dW"):
            assert torch.equal(ref[k], b[k]), (rep, k)
        assert float(junk) == float(junk)
