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


def _fp8_step(B, b, stream=None):
    B.cce_quantize_e4m3(b["H"], q=b["hq"], scales=b["hs"], stream=stream)
    B.cce_quantize_e4m3(b["W"], q=b["wq"], scales=b["wsc"], stream=stream)
    B.cce_fp8_forward(b["hq"], b["hs"], b["wq"], b["wsc"], b["y"], IGN, workspace=b["ws"], loss=b["loss"],
                      lse=b["lse"], stream=stream)
    B.cce_fp8_backward(b["hq"], b["hs"], b["wq"], b["wsc"], b["H"], b["W"], b["y"], b["lse"], b["dl"], IGN,
                       workspace=b["ws"], d_hidden=b["dH"], d_weight=b["dW"], stream=stream)


def _shard_step(B, b, stream=None):
    V = b["W"].shape[0]
    half = (V // 2) & ~7
    for p, (lo, hi) in enumerate([(0, half), (half, V)]):
        B.cce_shard_forward(b["H"], b["W"][lo:hi], b["y"], lo, stats=b["stats"][p], workspace=b["ws"], stream=stream)
    # the merge allocates its outputs in the binding; copy them into the fixed buffers
    loss, lse, _ = B.cce_shard_merge(b["stats"], b["y"], V, IGN, stream=stream)
    b["loss"].copy_(loss)
    b["lse"].copy_(lse)
    lo, hi = half, V
    B.cce_shard_backward(b["H"], b["W"][lo:hi], b["y"], b["lse"], b["dl"], lo, V, IGN, workspace=b["ws"],
                         d_hidden=b["dH"], d_weight=b["dW"][lo:hi], stream=stream)


def _compact_step(B, b, stream=None):
    B.cce_forward_compact(b["H"], b["W"], b["y"], b["n_valid"], IGN, workspace=b["wc"], loss=b["loss"], lse=b["lse"],
                          stream=stream)
    B.cce_backward_compact(b["H"], b["W"], b["y"], b["lse"], b["dl"], b["n_valid"], IGN, workspace=b["wc"],
                           d_hidden=b["dH"], d_weight=b["dW"], stream=stream)


@pytest.mark.parametrize("which", ["fp8", "shard", "compact"])
def test_graph_capture_of_the_variants(B, which):
    """The FP8 and the vocabulary-shard entry points are launches only as well: captured,
    replayed three times with eager work in between, every replay equal to the eager result."""
    w = I.make_workload(I.custom_spec(520, 256, 2100, seed=43, ignore_frac=0.1))
    step = {"fp8": _fp8_step, "shard": _shard_step, "compact": _compact_step}[which]
    B.set_row_skipping(2 if which == "compact" else 0)
    def buffers():
        b = _buffers(B, w)
        N, D = w.hidden.shape
        V = w.weight.shape[0]
        b["hq"] = torch.empty(N, D, dtype=torch.uint8, device="cuda")
        b["wq"] = torch.empty(V, D, dtype=torch.uint8, device="cuda")
        b["hs"] = torch.empty(B.fp8_scale_bytes(N, D), dtype=torch.uint8, device="cuda")
        b["wsc"] = torch.empty(B.fp8_scale_bytes(V, D), dtype=torch.uint8, device="cuda")
        b["stats"] = torch.empty(2, N, 4, device="cuda")
        b["n_valid"] = w.n_valid
        b["wc"] = B.alloc_compact_workspace(N, D, V, w.n_valid)
        b["dW"].zero_()
        return b
    ref, b = buffers(), buffers()
    step(B, ref)
    step(B, b)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            step(B, b, stream=s)
    for rep in range(3):
        for k in ("loss", "lse", "dH", "dW", "hq", "hs"):
            b[k].zero_()
        junk = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ("loss", "lse", "dH", "dW"):
            assert torch.equal(ref[k], b[k]), (which, rep, k)
        assert float(junk) == float(junk)
    B.set_row_skipping(0)


def test_two_host_threads_on_two_streams(B):
    """The library is called from more than one thread: two threads, each with its own stream, shapes,
    workspace and outputs, run forward + backward at the same time; every result equals what the same
    thread's inputs give when run alone.  (Plans are cached per thread, kernel set-up and the process-wide
    knobs are behind locks / atomics.)"""
    import threading
    specs = [I.custom_spec(700, 896, 3000, seed=45, ignore_frac=0.2), I.custom_spec(520, 256, 2100, seed=46, ignore_frac=0.1)]
    loads = [I.make_workload(sp) for sp in specs]
    refs = []
    for w in loads:
        r = _buffers(B, w)
        _step(B, r)
        refs.append(r)
    torch.cuda.synchronize()
    outs = [_buffers(B, w) for w in loads]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def worker(i):
        try:
            torch.cuda.set_device(0)
            for _ in range(6):
                for k in ("loss", "lse", "dH", "dW"):
                    outs[i][k].zero_()              # on the default stream of this thread's context: ordered below
                streams[i].wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(streams[i]):
                    _step(B, outs[i], stream=streams[i])
                streams[i].synchronize()
                for k in ("loss", "lse", "dH", "dW"):
                    if not torch.equal(refs[i][k], outs[i][k]):
                        errors.append((i, k))
        except Exception as exc:                    # surfaced in the main thread
            errors.append((i, repr(exc)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads)
    assert errors == []


def test_static_forward_under_graph_capture(B):
    """cce_forward_static is for callers that cannot allocate, code under graph capture among them:
    captured (after one call outside a capture), replayed three times with eager work in between, every
    replay equal to cce_forward."""
    w = I.make_workload(I.custom_spec(520, 128, 2100, seed=47, ignore_frac=0.1))
    H, W, y = dev_inputs(w)
    ref_loss, ref_lse = B.cce_forward(H, W, y, IGN)
    loss = torch.empty(520, device="cuda")
    lse = torch.empty(520, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.cce_forward_static(H, W, y, IGN, loss, lse, status)          # first use outside a capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            B.cce_forward_static(H, W, y, IGN, loss, lse, status, stream=s)
    for rep in range(3):
        loss.zero_()
        lse.zero_()
        status.fill_(77)
        junk = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss, ref_loss) and torch.equal(lse, ref_lse) and int(status.item()) == 0, rep
        assert float(junk) == float(junk)
