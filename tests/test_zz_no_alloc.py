"""The entry point that allocates nothing (lfmmi_forward_backward_static) against
lfmmi_forward_backward, through the C ABI: same arguments, the workspace in the
library's static device array. Two calls in a row, the second with a smaller
input, then the limits."""
import ctypes

import numpy as np
import pytest

from paper_2005_09824_amd import binding, workloads

pytestmark = pytest.mark.gpu

OBJF_RTOL = 1e-4
GRAD_ATOL = 1e-4


def _raw(entry, handle, x, lens, leak, scale, accumulate, objf, grad, status, stream):
    lib = binding.load_library()
    vp = ctypes.c_void_p
    B, T, P = x.shape
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    return getattr(lib, entry)(handle, vp(x.data_ptr()), lens.ctypes.data_as(vp), B, T, P,
                               float(leak), float(scale), int(accumulate), vp(objf.data_ptr()),
                               vp(grad.data_ptr()), vp(status.data_ptr()), vp(stream))


def _both(handle, logits, lens, leak, scale=1.0):
    """(static entry point's outputs, allocating entry point's outputs), as numpy."""
    import torch
    x = torch.from_numpy(np.ascontiguousarray(logits)).cuda()
    B, T, P = x.shape
    outs = []
    stream = torch.cuda.current_stream().cuda_stream
    for entry in ("lfmmi_forward_backward_static", "lfmmi_forward_backward"):
        objf = torch.full((B,), 7.0, dtype=torch.float32, device="cuda")
        grad = torch.full((B, T, P), -3.0, dtype=torch.float32, device="cuda")
        status = torch.full((B,), 9, dtype=torch.int32, device="cuda")
        rc = _raw(entry, handle.handle, x, lens, leak, scale, 0, objf, grad, status, stream)
        assert rc == 0, (entry, binding.lfmmi_last_error())
        torch.cuda.synchronize()
        outs.append((objf.cpu().numpy(), grad.cpu().numpy(), status.cpu().numpy()))
    return outs


def _same(got, want, lens):
    objf, grad, status = got
    objf_w, grad_w, status_w = want
    assert np.array_equal(status, status_w) and np.all(status == 0)
    assert np.all(np.abs(objf - objf_w) <= OBJF_RTOL * np.abs(objf_w))
    assert np.abs(grad - grad_w).max() <= GRAD_ATOL
    for b, Tb in enumerate(lens):
        assert np.all(grad[b, Tb:] == 0.0)
    # every sequence is computed by the same kernels in the same way
    assert np.array_equal(objf, objf_w) and np.array_equal(grad, grad_w)


def test_static_entry_point_equals_the_allocating_one_twice_in_a_row():
    # the first call: the metric's graph, ragged lengths, NaN in the padding frames;
    # the second, smaller one finds the first call's contents in the shared array
    wl = workloads.make_workload(2, scale={"B": 7, "Tlo": 30, "Thi": 120}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    got, want = _both(h, wl["logits"], wl["lengths"], wl["leak"])
    _same(got, want, wl["lengths"])
    small = workloads.make_workload(2, seed=99, scale={"B": 3, "Tlo": 5, "Thi": 40}, pad_value=np.nan)
    got, want = _both(h, small["logits"], small["lengths"], small["leak"], scale=-1.0)
    _same(got, want, small["lengths"])
    h.close()


def test_static_entry_point_numerator_batch_accumulate_and_limits():
    import torch
    # one graph per sequence (fp64 state vectors), then the denominator accumulated
    # on top: Eq. 2 / Eq. 3 through the static entry point alone
    wl = workloads.make_workload(5, scale={"S": 300, "B": 5, "nlo": 5, "nhi": 20}, pad_value=np.nan)
    x = torch.from_numpy(wl["logits"]).cuda()
    lens, leak = wl["lengths"], wl["leak"]
    B, T, P = x.shape
    num = binding.lfmmi_graph_create_batch(wl["num"])
    den = binding.lfmmi_graph_create(wl["den"])
    stream = torch.cuda.current_stream().cuda_stream
    res = []
    for entry in ("lfmmi_forward_backward_static", "lfmmi_forward_backward"):
        objf = torch.empty(B, dtype=torch.float32, device="cuda")
        grad = torch.empty((B, T, P), dtype=torch.float32, device="cuda")
        status = torch.empty(B, dtype=torch.int32, device="cuda")
        assert _raw(entry, num.handle, x, lens, leak, 1.0, 0, objf, grad, status, stream) == 0
        assert _raw(entry, den.handle, x, lens, leak, -1.0, 1, objf, grad, status, stream) == 0
        torch.cuda.synchronize()
        res.append((objf.cpu().numpy(), grad.cpu().numpy(), status.cpu().numpy()))
    assert np.all(res[0][2] == 0) and np.array_equal(res[0][2], res[1][2])
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])

    # limits: a clear error, nothing enqueued, outputs untouched
    unsupported = 5
    objf = torch.full((B,), 7.0, dtype=torch.float32, device="cuda")
    big_B = binding.STATIC_MAX_BATCH + 1
    xb = torch.zeros((big_B, 2, P), dtype=torch.float32, device="cuda")
    ob = torch.zeros(big_B, dtype=torch.float32, device="cuda")
    gb = torch.zeros((big_B, 2, P), dtype=torch.float32, device="cuda")
    sb = torch.zeros(big_B, dtype=torch.int32, device="cuda")
    rc = _raw("lfmmi_forward_backward_static", den.handle, xb, np.full(big_B, 2, np.int32), leak,
              1.0, 0, ob, gb, sb, stream)
    assert rc == unsupported and "sequences" in binding.lfmmi_last_error()
    # a workspace beyond the static array: 40 sequences of 2,000 frames on 320 + 320 rows
    Tl = 2000
    xl = torch.zeros((40, Tl, P), dtype=torch.float32, device="cuda")
    ol = torch.full((40,), 7.0, dtype=torch.float32, device="cuda")
    gl = torch.full((40, Tl, P), 7.0, dtype=torch.float32, device="cuda")
    sl = torch.zeros(40, dtype=torch.int32, device="cuda")
    rc = _raw("lfmmi_forward_backward_static", den.handle, xl, np.full(40, Tl, np.int32), leak,
              1.0, 0, ol, gl, sl, stream)
    assert rc == unsupported and "workspace" in binding.lfmmi_last_error()
    torch.cuda.synchronize()
    assert float(ol.min()) == 7.0 and float(gl.min()) == 7.0
    # the same handle still works through both entry points afterwards
    got, want = _both(den, wl["logits"], lens, leak)
    _same(got, want, lens)
    num.close(); den.close()


def test_static_entry_point_largest_batch_and_empty_sequences():
    # 256 sequences (the limit), unsorted lengths with zeros among them: descriptors
    # and launch order are written on the device from the lengths
    rng = np.random.default_rng(12)
    g = workloads.random_den_graph(rng, 150, 4, 20, 0.5)
    h = binding.lfmmi_graph_create(g)
    B = binding.STATIC_MAX_BATCH
    lens = rng.integers(0, 13, B).astype(np.int32)
    lens[[0, 17, 255]] = 0
    x = rng.normal(0, 2, (B, 12, 20)).astype(np.float32)
    for b in range(B):
        x[b, lens[b]:] = np.nan
    got, want = _both(h, x, lens, 1e-4)
    assert np.array_equal(got[2], want[2]) and np.all(got[2] == 0)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
    # T == 0: nothing to read, log Z of the empty sequence
    got, want = _both(h, np.zeros((3, 0, 20), np.float32), np.zeros(3, np.int32), 1e-4)
    assert np.array_equal(got[0], want[0]) and np.all(np.isfinite(got[0]))
    h.close()


def test_static_entry_point_under_hip_graph_capture():
    # the caller it is for: one call captured into a HIP graph (kernel launches only, on
    # the capturing stream) and replayed, with the program's own eager work and
    # synchronisations between the replays; every replay against the eager result
    import torch
    wl = workloads.make_workload(2, scale={"B": 6, "Tlo": 20, "Thi": 80}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    lens, leak = wl["lengths"], wl["leak"]
    x = torch.from_numpy(wl["logits"]).cuda()
    B, T, P = x.shape
    objf = torch.zeros(B, device="cuda")
    grad = torch.zeros((B, T, P), device="cuda")
    status = torch.zeros(B, dtype=torch.int32, device="cuda")
    ref = binding.lfmmi_forward_backward(h, x, lens, leak)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # once eagerly (first-use work stays out of the capture)
        binding.lfmmi_forward_backward_static(h, x, lens, leak, 1.0, False, objf, grad, status)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert torch.equal(objf, ref[0]) and torch.equal(grad, ref[1])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.lfmmi_forward_backward_static(h, x, lens, leak, 1.0, False, objf, grad, status)
    for _ in range(3):
        objf.fill_(7.0)
        grad.fill_(7.0)
        float((x[:, :5] * 2).nan_to_num().sum().item())   # eager work and a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(objf, ref[0]) and torch.equal(grad, ref[1])
        assert int(status.abs().sum().item()) == 0
    # other values in the same buffers: the replay reads them
    x2 = x.clone()
    x2[:, :10] *= 0.5
    ref2 = binding.lfmmi_forward_backward(h, x2, lens, leak)
    torch.cuda.synchronize()
    x.copy_(x2)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(objf, ref2[0]) and torch.equal(grad, ref2[1])
    del graph
    h.close()
