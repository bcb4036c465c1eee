"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.

Tolerances (fp32 path vs fp64 oracle): |objf - oracle| <= 1e-4 * |oracle|
(for num - den: 1e-4 * max(|num|, |den|, 1)), |grad - oracle| <= 1e-4 absolute.
"""
import numpy as np
import pytest

from oracle import lfmmi_oracle as oracle
from paper_2005_09824_amd import binding, workloads

pytestmark = pytest.mark.gpu

OBJF_RTOL = 1e-4
GRAD_ATOL = 1e-4


def _torch():
    import torch
    return torch


def run_gpu(handle, logits, lengths, leak, **kw):
    torch = _torch()
    x = torch.from_numpy(np.ascontiguousarray(logits)).cuda()
    objf, grad, status = binding.lfmmi_forward_backward(handle, x, lengths, leak, **kw)
    torch.cuda.synchronize()
    return objf.cpu().numpy(), grad.cpu().numpy(), status.cpu().numpy()


def check(objf, grad, status, lz, gamma, what=""):
    assert np.all(status == 0), (what, status)
    rel = np.abs(objf.astype(np.float64) - lz) / np.maximum(np.abs(lz), 1e-30)
    assert np.all(rel <= OBJF_RTOL), (what, "objf", rel.max())
    err = np.abs(grad.astype(np.float64) - gamma).max() if gamma.size else 0.0
    assert err <= GRAD_ATOL, (what, "grad", err)
    return float(rel.max()) if rel.size else 0.0, float(err)


def test_config1_denominator_numerators_and_full_loss():
    wl = workloads.make_workload(1, pad_value=np.nan)
    den = binding.lfmmi_graph_create(wl["den"])
    num = binding.lfmmi_graph_create_batch(wl["num"])
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    lz_d, g_d = oracle.forward_backward(wl["den"], x, lens, leak)
    lz_n, g_n = oracle.forward_backward_per_utt(wl["num"], x, lens, leak)
    rel_d, err_d = check(*run_gpu(den, x, lens, leak), lz_d, g_d, "den")
    rel_n, err_n = check(*run_gpu(num, x, lens, leak), lz_n, g_n, "num")
    print("config 1: objf max rel err %.2e, grad max abs err %.2e" % (max(rel_d, rel_n), max(err_d, err_n)))
    # Eq. 2 / Eq. 3: numerators with (+1, overwrite), denominator with (-1, accumulate)
    torch = _torch()
    xd = torch.from_numpy(x).cuda()
    objf, grad, status = binding.lfmmi_forward_backward(num, xd, lens, leak, 1.0, False)
    binding.lfmmi_forward_backward(den, xd, lens, leak, -1.0, True, objf, grad, status)
    torch.cuda.synchronize()
    objf, grad = objf.cpu().numpy().astype(np.float64), grad.cpu().numpy().astype(np.float64)
    tol = OBJF_RTOL * np.maximum(np.maximum(np.abs(lz_n), np.abs(lz_d)), 1.0)
    assert np.all(np.abs(objf - (lz_n - lz_d)) <= tol)
    assert np.abs(grad - (g_n - g_d)).max() <= GRAD_ATOL
    assert np.all(status.cpu().numpy() == 0)
    den.close(); num.close()


@pytest.mark.parametrize("config,scale", [
    (2, {"S": 300, "B": 5, "Tlo": 30, "Thi": 70}),          # several slices, ragged tail
    (2, {"S": 2000, "B": 3, "Tlo": 20, "Thi": 40}),          # the metric's graph, short
    (3, {"S": 700, "P": 300, "B": 4, "Tlo": 20, "Thi": 50}),  # Zipf pdfs, P > 256
    (4, {"S": 500, "B": 4, "Tlo": 100, "Thi": 400}),         # unsorted lengths, +-30 spikes
])
def test_scaled_configs_every_element(config, scale):
    wl = workloads.make_workload(config, scale=scale, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    lz, gamma = oracle.forward_backward(wl["den"], wl["logits"], wl["lengths"], wl["leak"])
    out = run_gpu(h, wl["logits"], wl["lengths"], wl["leak"])
    check(*out, lz, gamma, "config %d scaled" % config)
    # padded rows are exactly zero and valid rows sum to one
    for b, Tb in enumerate(wl["lengths"]):
        assert np.all(out[1][b, Tb:] == 0.0)
        assert np.allclose(out[1][b, :Tb].sum(1), 1.0, atol=2e-4)
    h.close()


def test_nonuniform_start_distribution_on_the_register_path():
    # a start distribution that is not uniform: every arc carries its leak factor
    # and slices end in closing slots; all final weights positive keeps it in fp32
    wl = workloads.make_workload(2, scale={"S": 1500, "B": 4, "Tlo": 20, "Thi": 45}, pad_value=np.nan)
    g = wl["den"]
    rng = np.random.default_rng(7)
    pi = rng.uniform(0.05, 1.0, g["num_states"])
    g["init_prob"] = (pi / pi.sum()).astype(np.float32)
    g["final_prob"] = rng.uniform(0.2, 1.0, g["num_states"]).astype(np.float32)
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["per_arc_leak"] == 1 and info["closing_slots"] == 1 and info["register_slots"] > 0
    assert binding.lfmmi_graph_info(h)["fp64"] == 0
    lz, gamma = oracle.forward_backward(g, wl["logits"], wl["lengths"], wl["leak"])
    check(*run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]), lz, gamma, "non-uniform pi")
    h.close()


def test_graph_too_large_for_the_registers_keeps_part_of_each_wave_there():
    # config 4's graph: more arcs per wave than any register-resident variant holds;
    # the first slots of a wave stay in registers, the others are streamed
    wl = workloads.make_workload(4, scale={"B": 3, "Tlo": 9, "Thi": 40}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    for o in (0, 1):
        info = binding.lfmmi_graph_ordering_info(h, 0, o)
        assert 0 < info["register_slots"] < info["max_wave_slots"]
    lz, gamma = oracle.forward_backward(wl["den"], wl["logits"], wl["lengths"], wl["leak"])
    check(*run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]), lz, gamma, "hybrid")
    h.close()


def test_large_graph_keeps_part_of_each_wave_in_registers_too():
    # config 3's graph: more than 8192 states (48 KB state vectors in LDS)
    wl = workloads.make_workload(3, scale={"B": 2, "Tlo": 8, "Thi": 25}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["rows"] > 8192 and 0 < info["register_slots"] < info["max_wave_slots"]
    lz, gamma = oracle.forward_backward(wl["den"], wl["logits"], wl["lengths"], wl["leak"])
    check(*run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]), lz, gamma, "hybrid, large map")
    h.close()


@pytest.mark.parametrize("frames,groups", [(1, 1), (1, 4), (2, 1), (2, 2), (2, 3)])
def test_occupancy_kernel_with_one_or_two_frames_per_arc_record(frames, groups, monkeypatch):
    # config 4's graph (5,056 padded rows: 32 KB planes in LDS): one frame per arc record, or
    # two with the second pair of planes beyond 64 KB; odd lengths leave the last group half
    # empty, and a length of 1 leaves a workgroup's later groups without any frame
    monkeypatch.setenv("LFMMI_OCC_MULTI", str(frames))
    monkeypatch.setenv("LFMMI_OCC_GROUPS", str(groups))
    wl = workloads.make_workload(4, scale={"B": 5, "Tlo": 40, "Thi": 40})
    lengths = np.array([37, 1, 24, 9, 40], dtype=wl["lengths"].dtype)
    logits = wl["logits"].copy()
    for b, Tb in enumerate(lengths):
        logits[b, Tb:] = np.nan
    h = binding.lfmmi_graph_create(wl["den"])
    lz, gamma = oracle.forward_backward(wl["den"], logits, lengths, wl["leak"])
    out = run_gpu(h, logits, lengths, wl["leak"])
    check(*out, lz, gamma, "occupancy, %d frame(s) per record, %d group(s)" % (frames, groups))
    for b, Tb in enumerate(lengths):
        assert np.all(out[1][b, Tb:] == 0.0)
    h.close()


def test_occupancy_wave_with_more_slices_than_it_keeps_places_for():
    # 2,500 pdfs on a 1,500-state graph: 40 slices of occupancy rows for 8 waves, five each;
    # the four-frame kernel keeps the places of a wave's first four slices in registers and
    # fetches the fifth's when that slice ends
    rng = np.random.default_rng(5)
    g = workloads.random_den_graph(rng, 1500, 19, 2500, 0.5, "uniform")
    lengths = np.array([23, 9, 16], np.int32)
    x = rng.normal(0, 2, (3, 23, 2500)).astype(np.float32)
    for b, Tb in enumerate(lengths):
        x[b, Tb:] = np.nan
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 2)
    assert info["waves"] == 8 and info["slices"] >= 5 * 8
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "five occupancy slices per wave")
    h.close()


def test_largest_graph_the_library_takes():
    # 16,384 states, the limit: state vectors of 64 KB each, streamed arcs, the
    # frame-at-a-time occupancy kernel; one state more is refused when the graph is made
    rng = np.random.default_rng(99)
    g = workloads.random_den_graph(rng, 16384, 3, 200, 0.5, "uniform")
    lengths = np.array([11, 6], np.int32)
    x = rng.normal(0, 2, (2, 11, 200)).astype(np.float32)
    x[1, 6:] = np.nan
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["rows"] == 16384 and info["register_slots"] == 0
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "16384 states")
    h.close()
    g2 = workloads.random_den_graph(rng, 16385, 2, 200, 0.5, "uniform")
    with pytest.raises(binding.LfmmiError) as err:
        binding.lfmmi_graph_create(g2)
    assert "16384" in str(err.value)


def test_wave_with_more_than_64_streamed_slices(monkeypatch):
    # two waves for 141 slices: each streams about 70 slices a frame, more than the
    # 64 whose ends (and hub flags) a wave keeps in the lanes of one register
    monkeypatch.setenv("LFMMI_WAVES", "2")
    rng = np.random.default_rng(4242)
    g = workloads.random_den_graph(rng, 9000, 3, 300, 0.5, "uniform")
    lengths = np.array([7, 12], np.int32)
    x = rng.normal(0, 2, (2, 12, 300)).astype(np.float32)
    x[0, 7:] = np.nan
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["waves"] == 2 and 0 < info["register_slots"] < info["max_wave_slots"]
    assert info["slices"] > 2 * 64 + 2
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "two waves")
    h.close()


def test_pdf_with_many_occupancy_rows_fp32_and_fp64():
    # one pdf on most arcs: its arc list is cut into many rows, whose sums a whole
    # wave adds up; with some final weights zero the graph runs in fp64
    wl = workloads.make_workload(3, scale={"S": 600, "P": 40, "B": 3, "Tlo": 15, "Thi": 40},
                                 pad_value=np.nan)
    g = wl["den"]
    rng = np.random.default_rng(11)
    pdf = g["pdf"].copy()
    pdf[rng.random(len(pdf)) < 0.6] = 5
    g["pdf"] = pdf
    for fp64 in (0, 1):
        if fp64:
            fin = g["final_prob"].copy()
            fin[rng.random(len(fin)) < 0.5] = 0.0
            g["final_prob"] = fin
        h = binding.lfmmi_graph_create(g)
        assert binding.lfmmi_graph_info(h)["fp64"] == fp64
        oc = binding.lfmmi_graph_ordering_copy(h, 0, binding.ORD_OCC)
        assert np.count_nonzero(oc["row_id"] == 5) > 64
        lz, gamma = oracle.forward_backward(g, wl["logits"], wl["lengths"], wl["leak"])
        check(*run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]), lz, gamma, "heavy pdf")
        h.close()


@pytest.mark.parametrize("S,k,P,dist,nonuniform_pi,zero_finals,B,Tlo,Thi,expect", [
    (3000, 14, 200, "uniform", 0, 0, 3, 10, 30, "hybrid"),     # 32 KB state vectors, replicated emission row
    (3000, 14, 1200, "zipf", 0, 0, 3, 10, 30, "hybrid"),       # plain emission row, pdfs with many rows
    (9000, 6, 3500, "uniform", 0, 0, 2, 8, 20, "streamed"),    # more pdfs than the staging of the register paths takes
    (3000, 14, 100, "uniform", 1, 0, 3, 10, 30, "streamed"),   # per-arc leak factors, too many arcs for registers
    (1500, 10, 60, "uniform", 1, 1, 3, 10, 30, "fp64"),        # fp64 with per-arc leak factors
    (2500, 12, 90, "zipf", 0, 1, 3, 10, 30, "fp64"),           # fp64, larger
    (5000, 3, 84, "uniform", 0, 0, 3, 10, 30, "registers"),    # sparse rows
    (700, 30, 50, "uniform", 0, 0, 3, 10, 30, "some_registers"),  # dense rows: one wide slice per wave
    (13000, 3, 300, "uniform", 0, 0, 2, 6, 12, "streamed"),    # more states than the fixed LDS maps hold
    (64, 5, 7, "uniform", 0, 0, 5, 1, 9, "registers"),         # one slice, lengths from 1
])
def test_odd_shapes_through_every_recursion_variant(S, k, P, dist, nonuniform_pi, zero_finals,
                                                    B, Tlo, Thi, expect):
    rng = np.random.default_rng(1000 + S + P)
    g = workloads.random_den_graph(rng, S, k, P, 0.5, dist)
    if nonuniform_pi:
        pi = rng.uniform(0.05, 1.0, S)
        g["init_prob"] = (pi / pi.sum()).astype(np.float32)
    if zero_finals:
        fin = g["final_prob"].copy()
        fin[rng.random(S) < 0.6] = 0.0
        fin[0] = 1.0
        g["final_prob"] = fin
    lengths = rng.integers(Tlo, Thi + 1, B).astype(np.int32)
    T = int(lengths.max())
    x = rng.normal(0, 2, (B, T, P)).astype(np.float32)
    for b in range(B):
        x[b, lengths[b]:] = np.nan
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    fp64 = binding.lfmmi_graph_info(h)["fp64"]
    if expect == "fp64":
        assert fp64 == 1
    else:
        assert fp64 == 0
        if expect == "registers":
            assert info["register_slots"] >= info["max_wave_slots"]
        elif expect == "hybrid":
            assert 0 < info["register_slots"] < info["max_wave_slots"]
        elif expect == "some_registers":
            assert info["register_slots"] > 0
        else:
            assert info["register_slots"] == 0
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "S %d P %d %s" % (S, P, expect))
    h.close()


def test_concurrent_buckets_do_not_change_any_bit(monkeypatch):
    # sequences are cut by length into buckets that run on streams of their own;
    # every sequence is computed the same way whichever bucket it lands in
    wl = workloads.make_workload(2, scale={"S": 400, "B": 13, "Tlo": 5, "Thi": 90}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    outs = []
    for buckets in ("1", "2", "4"):
        monkeypatch.setenv("LFMMI_BUCKETS", buckets)
        outs.append(run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]))
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and np.array_equal(o[1], outs[0][1])
        assert np.array_equal(o[2], outs[0][2])
    lz, gamma = oracle.forward_backward(wl["den"], wl["logits"], wl["lengths"], wl["leak"])
    check(*outs[-1], lz, gamma, "4 buckets")
    h.close()


def test_config5_scaled_full_loss():
    wl = workloads.make_workload(5, scale={"S": 400, "B": 6, "nlo": 5, "nhi": 25})
    den = binding.lfmmi_graph_create(wl["den"])
    num = binding.lfmmi_graph_create_batch(wl["num"])
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    lz_n, g_n = oracle.forward_backward_per_utt(wl["num"], x, lens, leak)
    lz_d, g_d = oracle.forward_backward(wl["den"], x, lens, leak)
    want_objf, want_grad = lz_n - lz_d, g_n - g_d
    check(*run_gpu(num, x, lens, leak), lz_n, g_n, "num")
    o_d = run_gpu(den, x, lens, leak)
    check(*o_d, lz_d, g_d, "den")
    torch = _torch()
    xd = torch.from_numpy(x).cuda()
    objf, grad, status = binding.lfmmi_forward_backward(num, xd, lens, leak, 1.0, False)
    binding.lfmmi_forward_backward(den, xd, lens, leak, -1.0, True, objf, grad, status)
    torch.cuda.synchronize()
    tol = OBJF_RTOL * np.maximum(np.maximum(np.abs(lz_n), np.abs(lz_d)), 1.0)
    assert np.all(np.abs(objf.cpu().numpy().astype(np.float64) - want_objf) <= tol)
    assert np.abs(grad.cpu().numpy().astype(np.float64) - want_grad).max() <= GRAD_ATOL
    den.close(); num.close()


def test_edge_cases_lengths_zero_empty_batch_and_leak_zero():
    torch = _torch()
    wl = workloads.make_workload(2, scale={"S": 130, "B": 4, "Tlo": 3, "Thi": 9})
    g = wl["den"]
    g["init_prob"] = np.random.default_rng(0).uniform(0, 1, 130).astype(np.float32)
    g["final_prob"] = np.random.default_rng(1).uniform(0, 1, 130).astype(np.float32)
    h = binding.lfmmi_graph_create(g)
    lens = wl["lengths"].copy()
    lens[1] = 0                       # an empty sequence: log Z = log(f^T L pi)
    lens[2] = 1
    for leak in (0.0, 1e-5, 0.25):
        lz, gamma = oracle.forward_backward(g, wl["logits"], lens, leak)
        check(*run_gpu(h, wl["logits"], lens, leak), lz, gamma, "leak %g" % leak)
    # B = 0 and T = 0
    x0 = torch.zeros((0, 4, 84), dtype=torch.float32, device="cuda")
    binding.lfmmi_forward_backward(h, x0, np.zeros(0, np.int32), 1e-5)
    x1 = torch.zeros((2, 0, 84), dtype=torch.float32, device="cuda")
    objf, grad, status = binding.lfmmi_forward_backward(h, x1, np.zeros(2, np.int32), 1e-5)
    torch.cuda.synchronize()
    lz, _ = oracle.forward_backward(g, np.zeros((2, 0, 84), np.float32), np.zeros(2, np.int32), 1e-5)
    assert np.allclose(objf.cpu().numpy(), lz, rtol=1e-5)
    h.close()


def test_dead_sequences_and_nonfinite_logits_are_flagged():
    # a chain that needs exactly 5 frames: T = 4 has zero probability without a leak
    K, P = 6, 3
    src = np.arange(K - 1, dtype=np.int32)
    g = {"num_states": K, "num_pdfs": P, "src": src, "dst": src + 1,
         "pdf": (src % P).astype(np.int32), "logw": np.zeros(K - 1, np.float32),
         "init_prob": np.eye(K, dtype=np.float32)[0], "final_prob": np.eye(K, dtype=np.float32)[K - 1]}
    h = binding.lfmmi_graph_create(g)
    rng = np.random.default_rng(5)
    x = rng.normal(size=(3, 5, P)).astype(np.float32)
    lens = np.array([5, 4, 5], dtype=np.int32)
    x[2, 3, 1] = np.nan
    objf, grad, status = run_gpu(h, x, lens, 0.0)
    lz, gamma = oracle.forward_backward(g, x[:1], lens[:1], 0.0)
    assert status.tolist() == [0, 1, 3]
    assert abs(objf[0] - lz[0]) <= OBJF_RTOL * abs(lz[0])
    assert np.abs(grad[0] - gamma[0]).max() <= GRAD_ATOL
    assert objf[1] == -np.inf and np.isnan(objf[2])
    assert np.all(grad[1:] == 0.0)
    h.close()


def test_sequence_result_does_not_depend_on_batch_neighbours():
    wl = workloads.make_workload(2, scale={"S": 200, "B": 6, "Tlo": 10, "Thi": 30})
    h = binding.lfmmi_graph_create(wl["den"])
    full = run_gpu(h, wl["logits"], wl["lengths"], wl["leak"])
    perm = np.array([3, 0, 5, 1, 4, 2])
    part = run_gpu(h, wl["logits"][perm], wl["lengths"][perm], wl["leak"])
    assert np.allclose(full[0][perm], part[0], rtol=1e-6)
    assert np.allclose(full[1][perm], part[1], atol=1e-6)
    h.close()


# ---- the five workloads at full size, in the launch configuration bench.py times:
# every objective and every gradient entry of the whole batch against the oracle,
# and the properties that hold at any size on every sequence.
def _full_size(config, sample):
    wl = workloads.make_workload(config)
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    den = binding.lfmmi_graph_create(wl["den"])
    objf, grad, status = run_gpu(den, x, lens, leak)
    assert np.all(status == 0)
    assert np.all(np.isfinite(objf))
    for b, Tb in enumerate(lens):
        assert np.all(grad[b, Tb:] == 0.0)
        rows = grad[b, :Tb].astype(np.float64).sum(1)
        assert np.abs(rows - 1.0).max() <= 2e-4, (b, np.abs(rows - 1.0).max())
        assert grad[b, :Tb].min() >= 0.0
    idx = np.asarray(sample)
    lz, gamma = oracle.forward_backward(wl["den"], x[idx], lens[idx], leak)
    rel, err = check(objf[idx], grad[idx], status[idx], lz, gamma, "config %d" % config)
    print("config %d full size: objf max rel err %.2e, grad max abs err %.2e" % (config, rel, err))
    den.close()
    return wl


def test_config2_full_size_all_sequences():
    _full_size(2, list(range(64)))


def test_config3_full_size_all_sequences():
    _full_size(3, list(range(128)))


def test_config4_full_size_all_sequences():
    _full_size(4, list(range(32)))


def test_config5_full_size_all_sequences():
    wl = workloads.make_workload(5)
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    torch = _torch()
    den = binding.lfmmi_graph_create(wl["den"])
    num = binding.lfmmi_graph_create_batch(wl["num"])
    lz_n, g_n = oracle.forward_backward_per_utt(wl["num"], x, lens, leak)
    check(*run_gpu(num, x, lens, leak), lz_n, g_n, "config 5 numerators")
    xd = torch.from_numpy(x).cuda()
    objf, grad, status = binding.lfmmi_forward_backward(num, xd, lens, leak, 1.0, False)
    binding.lfmmi_forward_backward(den, xd, lens, leak, -1.0, True, objf, grad, status)
    torch.cuda.synchronize()
    objf, grad = objf.cpu().numpy().astype(np.float64), grad.cpu().numpy().astype(np.float64)
    assert np.all(status.cpu().numpy() == 0)
    for b, Tb in enumerate(lens):   # gamma_num and gamma_den each sum to one per frame
        assert np.abs(grad[b, :Tb].sum(1)).max() <= 4e-4
        assert np.all(grad[b, Tb:] == 0.0)
    lz_d, g_d = oracle.forward_backward(wl["den"], x, lens, leak)
    tol = OBJF_RTOL * np.maximum(np.maximum(np.abs(lz_n), np.abs(lz_d)), 1.0)
    err_o = np.abs(objf - (lz_n - lz_d))
    assert np.all(err_o <= tol)
    err_g = np.abs(grad - (g_n - g_d)).max()
    assert err_g <= GRAD_ATOL
    print("config 5 full size: objf max err / tolerance %.2e, grad max abs err %.2e"
          % ((err_o / tol).max(), err_g))
    den.close(); num.close()


def test_a_call_with_its_four_buckets_replays_from_a_hip_graph():
    # after one eager call (workspace allocated, descriptors staged) a call enqueues kernels,
    # event records and event waits only: captured on a side stream, with the buckets' streams
    # joining the capture through the fork event, it replays with the same bits, also with
    # eager calls and synchronisations between the replays
    torch = _torch()
    wl = workloads.make_workload(2, scale={"S": 600, "B": 12, "Tlo": 20, "Thi": 90})
    h = binding.lfmmi_graph_create(wl["den"])
    x = torch.from_numpy(wl["logits"]).cuda()
    B, T, P = x.shape
    objf = torch.empty(B, device="cuda")
    grad = torch.empty((B, T, P), device="cuda")
    status = torch.zeros(B, dtype=torch.int32, device="cuda")

    def call():
        binding.lfmmi_forward_backward(h, x, wl["lengths"], wl["leak"], 1.0, False, objf, grad, status)

    call()
    torch.cuda.synchronize()
    want_o, want_g = objf.clone(), grad.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side, capture_error_mode="relaxed"):
            call()
    torch.cuda.synchronize()
    for _ in range(3):
        objf.zero_()
        grad.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(objf, want_o) and torch.equal(grad, want_g)
        call()                      # eager work between the replays
        torch.cuda.synchronize()
    assert int(status.abs().max()) == 0
    del graph
    h.close()


def test_autograd_wrapper_gives_the_objective_and_its_gradient():
    torch = _torch()
    from paper_2005_09824_amd import chain
    wl = workloads.make_workload(5, scale={"S": 300, "B": 5, "nlo": 4, "nhi": 12})
    den = binding.lfmmi_graph_create(wl["den"])
    num = binding.lfmmi_graph_create_batch(wl["num"])
    x = torch.from_numpy(wl["logits"]).cuda().requires_grad_(True)
    loss = chain.chain_loss(x, wl["lengths"], num, den, wl["leak"])
    loss.backward()
    torch.cuda.synchronize()
    want_objf, want_grad, lz_n, lz_d = oracle.loss(wl["num"], wl["den"], wl["logits"],
                                                   wl["lengths"], wl["leak"])
    frames = float(wl["lengths"].sum())
    tol = 1e-4 * np.maximum(np.maximum(np.abs(lz_n), np.abs(lz_d)), 1.0).sum() / frames
    assert abs(float(loss.item()) - (-want_objf.sum() / frames)) <= tol
    assert np.abs(x.grad.cpu().numpy().astype(np.float64) * (-frames) - want_grad).max() <= GRAD_ATOL
    den.close(); num.close()


def test_profiling_levels_report_launch_durations_and_leave_results_alone():
    wl = workloads.make_workload(2, scale={"S": 300, "B": 6, "Tlo": 20, "Thi": 60}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    plain = run_gpu(h, wl["logits"], wl["lengths"], wl["leak"])
    for level, timed in ((1, ("emit", "rec", "occ")), (2, ("rec",))):
        binding.lfmmi_profile_enable(h, level)
        outs = [run_gpu(h, wl["logits"], wl["lengths"], wl["leak"]) for _ in range(2)]
        with pytest.raises(binding.LfmmiError):  # recorded calls must be read first
            binding.lfmmi_profile_enable(h, 3 - level)
        pr = binding.lfmmi_profile_read(h)
        binding.lfmmi_profile_enable(h, 0)
        assert pr["calls"] == 2 and pr["launches"] >= 2
        for k in ("emit", "rec", "occ"):
            assert (pr[k] > 0.0) == (k in timed), (level, pr)
        for o in outs:
            assert np.array_equal(o[0], plain[0]) and np.array_equal(o[1], plain[1])
    with pytest.raises(binding.LfmmiError):
        binding.lfmmi_profile_read(h)  # nothing recorded
    with pytest.raises(binding.LfmmiError):
        binding.lfmmi_profile_enable(h, 7)
    h.close()


def test_raw_call_without_status_on_a_side_stream_and_argument_errors():
    # the C entry point itself: status may be NULL, the stream is the caller's, and
    # bad arguments come back as status codes before anything is enqueued
    import ctypes
    torch = _torch()
    wl = workloads.make_workload(2, scale={"S": 300, "B": 4, "Tlo": 20, "Thi": 50}, pad_value=np.nan)
    h = binding.lfmmi_graph_create(wl["den"])
    ref = run_gpu(h, wl["logits"], wl["lengths"], wl["leak"])
    lib = binding.load_library()
    x = torch.from_numpy(wl["logits"]).cuda()
    B, T, P = x.shape
    lens = np.ascontiguousarray(wl["lengths"], dtype=np.int32)
    objf = torch.full((B,), 7.0, dtype=torch.float32, device="cuda")
    grad = torch.full((B, T, P), 7.0, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    vp = ctypes.c_void_p

    def call(handle=h.handle, logits=x.data_ptr(), lengths=lens, b=B, t=T, p=P, leak=wl["leak"],
             scale=1.0, objf_ptr=objf.data_ptr(), grad_ptr=grad.data_ptr()):
        return lib.lfmmi_forward_backward(handle, vp(logits), lengths.ctypes.data_as(vp), b, t, p,
                                          float(leak), float(scale), 0, vp(objf_ptr), vp(grad_ptr),
                                          vp(None), vp(side.cuda_stream))

    side.wait_stream(torch.cuda.current_stream())
    assert call() == 0
    side.synchronize()
    assert np.array_equal(objf.cpu().numpy(), ref[0]) and np.array_equal(grad.cpu().numpy(), ref[1])

    invalid = 1
    assert call(p=P + 1) == invalid and "num_pdfs" in binding.lfmmi_last_error()
    assert call(b=-1) == invalid
    assert call(leak=-1.0) == invalid and call(leak=float("nan")) == invalid
    assert call(scale=float("nan")) == invalid
    assert call(lengths=np.array([T + 1] * B, np.int32)) == invalid
    assert call(lengths=np.array([-1] * B, np.int32)) == invalid
    assert call(logits=0) == invalid and call(objf_ptr=0) == invalid and call(grad_ptr=0) == invalid
    assert call(handle=None) == invalid
    assert call(b=0) == 0  # an empty batch is valid and enqueues nothing
    packed_only = binding.lfmmi_graph_pack(wl["den"])
    assert call(handle=packed_only.handle) == invalid and "uploaded" in binding.lfmmi_last_error()
    packed_only.close()
    # a batch handle needs one graph per sequence
    nums = workloads.make_workload(1, pad_value=np.nan)["num"]
    nb = binding.lfmmi_graph_create_batch(nums)
    with pytest.raises(binding.LfmmiError):
        binding.lfmmi_forward_backward(nb, torch.zeros((len(nums) + 1, 4, 10), device="cuda"),
                                       np.full(len(nums) + 1, 4, np.int32), 1e-5)
    nb.close()
    # the outputs of the good call were not touched by the refused ones
    torch.cuda.synchronize()
    assert np.array_equal(grad.cpu().numpy(), ref[1])
    h.close()


def test_loss_call_equals_the_two_passes_bit_for_bit_and_the_oracle():
    # Eq. 2 / Eq. 3 in one call
    torch = _torch()
    for seed, scale in ((3, {"S": 400, "B": 9, "Tlo": 12, "Thi": 70}), (4, {"B": 5, "Tlo": 40, "Thi": 90})):
        wl = workloads.make_workload(5, seed=seed, scale=scale, pad_value=np.nan)
        x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
        den = binding.lfmmi_graph_create(wl["den"])
        num = binding.lfmmi_graph_create_batch(wl["num"])
        xd = torch.from_numpy(x).cuda()
        objf2, grad2, st2 = binding.lfmmi_forward_backward(num, xd, lens, leak, 1.0, False)
        binding.lfmmi_forward_backward(den, xd, lens, leak, -1.0, True, objf2, grad2, st2)
        torch.cuda.synchronize()
        # stale contents of the outputs must not matter; two calls in a row
        objf = torch.full_like(objf2, 7.0); grad = torch.full_like(grad2, -3.0)
        st = torch.full_like(st2, 5)
        for _ in range(2):
            binding.lfmmi_loss(num, den, xd, lens, leak, objf, grad, st)
        torch.cuda.synchronize()
        assert torch.equal(objf, objf2) and torch.equal(grad, grad2) and torch.equal(st, st2)
        lz_n, g_n = oracle.forward_backward_per_utt(wl["num"], x, lens, leak)
        lz_d, g_d = oracle.forward_backward(wl["den"], x, lens, leak)
        tol = OBJF_RTOL * np.maximum(np.maximum(np.abs(lz_n), np.abs(lz_d)), 1.0)
        assert np.all(np.abs(objf.cpu().numpy().astype(np.float64) - (lz_n - lz_d)) <= tol)
        assert np.abs(grad.cpu().numpy().astype(np.float64) - (g_n - g_d)).max() <= GRAD_ATOL
        assert np.all(st.cpu().numpy() == 0)
        # status None, and a flagged sequence: non-finite logits reach both passes
        xb = x.copy(); xb[1, 3, 2] = np.inf
        o3, g3, s3 = binding.lfmmi_loss(num, den, torch.from_numpy(xb).cuda(), lens, leak)
        torch.cuda.synchronize()
        s3 = s3.cpu().numpy()
        assert s3[1] & 2 and np.all(np.delete(s3, 1) == 0) and np.isnan(o3.cpu().numpy()[1])
        with pytest.raises(binding.LfmmiError):
            binding.lfmmi_loss(den, den, xd, lens, leak)
        den.close(); num.close()


def _with_hubs(g, rng, in_hub, out_hub):
    S, P = g["num_states"], g["num_pdfs"]
    src = rng.choice(S, size=in_hub, replace=False).astype(np.int32)
    dst = rng.choice(S, size=out_hub, replace=False).astype(np.int32)
    g["src"] = np.concatenate([g["src"], src, np.full(out_hub, 3, np.int32)])
    g["dst"] = np.concatenate([g["dst"], np.full(in_hub, 5, np.int32), dst])
    n = in_hub + out_hub
    g["pdf"] = np.concatenate([g["pdf"], rng.integers(0, P, n).astype(np.int32)])
    g["logw"] = np.concatenate([g["logw"], np.log(rng.uniform(0.01, 0.2, n)).astype(np.float32)])
    return g


@pytest.mark.parametrize("kind", ["registers", "hybrid", "nonuniform_pi", "fp64", "fp64_registers"])
def test_hub_states_in_every_recursion_variant(kind):
    # a state with hundreds of arcs gets a slice of its own whose 64 lanes share its
    # arcs; the lanes' sums are added up where the slice ends
    rng = np.random.default_rng(21)
    if kind == "hybrid":
        g = workloads.random_den_graph(rng, 3000, 14, 60, 0.5)
    elif kind == "fp64_registers":
        g = workloads.random_den_graph(rng, 400, 3, 60, 0.5)
    else:
        g = workloads.random_den_graph(rng, 900, 8, 60, 0.5)
    g = _with_hubs(g, rng, *((150, 120) if kind == "fp64_registers" else (500, 350)))
    if kind in ("nonuniform_pi", "fp64", "fp64_registers"):
        pi = rng.uniform(0.05, 1.0, g["num_states"])
        g["init_prob"] = (pi / pi.sum()).astype(np.float32)
    if kind in ("fp64", "fp64_registers"):
        fin = g["final_prob"].copy()
        fin[rng.random(len(fin)) < 0.5] = 0.0
        fin[5] = 1.0
        g["final_prob"] = fin
    B = 4
    lengths = rng.integers(8, 40, B).astype(np.int32)
    x = rng.normal(0, 2, (B, int(lengths.max()), 60)).astype(np.float32)
    for b in range(B):
        x[b, lengths[b]:] = np.nan
    h = binding.lfmmi_graph_create(g)
    for o in (0, 1):
        info = binding.lfmmi_graph_ordering_info(h, 0, o)
        assert info["hub_slices"] == 1
        if kind in ("registers", "fp64_registers"):
            assert info["register_slots"] >= info["max_wave_slots"]
        if kind == "hybrid":
            assert 0 < info["register_slots"] < info["max_wave_slots"]
    assert binding.lfmmi_graph_info(h)["fp64"] == (1 if kind.startswith("fp64") else 0)
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "hubs, " + kind)
    h.close()


def test_many_hub_slices_push_the_padded_rows_past_the_fixed_lds_map():
    # 8000 states fit the 32 KB state vectors of the register-resident kernels, the
    # 8000 + 9 * 63 padded rows of nine hub slices do not: the kernel is chosen by
    # rows, and every element still matches
    rng = np.random.default_rng(77)
    S, P, deg = 8000, 84, 500
    g = workloads.random_den_graph(rng, S, 9, P, 0.5)
    src, dst = [g["src"]], [g["dst"]]
    for hub in range(9):
        src.append(rng.choice(S, size=deg, replace=False).astype(np.int32))
        dst.append(np.full(deg, 100 + hub, np.int32))
    for hub in range(2):
        src.append(np.full(deg, 4000 + hub, np.int32))
        dst.append(rng.choice(S, size=deg, replace=False).astype(np.int32))
    n = 11 * deg
    g["src"], g["dst"] = np.concatenate(src), np.concatenate(dst)
    g["pdf"] = np.concatenate([g["pdf"], rng.integers(0, P, n).astype(np.int32)])
    g["logw"] = np.concatenate([g["logw"], np.log(rng.uniform(0.001, 0.01, n)).astype(np.float32)])
    lengths = np.array([14, 9, 20], np.int32)
    x = rng.normal(0, 2, (3, 20, P)).astype(np.float32)
    for b in range(3):
        x[b, lengths[b]:] = np.nan
    h = binding.lfmmi_graph_create(g)
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["hub_slices"] == 9 and info["slices"] * 64 > 8192
    assert info["register_slots"] == 0 or info["slices"] * 64 <= info["lds_vector_rows"]
    lz, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    check(*run_gpu(h, x, lengths, 1e-5), lz, gamma, "many hubs")
    h.close()


def _left_to_right(rng, n_phones, P, all_initial):
    """The numerator topology (two states per phone, optional silence) with every
    state final; a unique start state, or every state initial."""
    g = workloads.phone_string_num_graph(rng.integers(1, 42, size=n_phones), P, 0.2)
    g["final_prob"] = np.ones(g["num_states"], np.float32)
    if all_initial:
        g["init_prob"] = np.full(g["num_states"], 1.0 / g["num_states"], np.float32)
    return g


def _match_or_flagged(out, lz, gamma, lens):
    """Every sequence either agrees with the oracle or carries a status flag."""
    objf, grad, status = out
    ok = 0
    for b in range(len(lens)):
        if status[b] != 0:
            continue
        assert abs(objf[b] - lz[b]) <= OBJF_RTOL * max(abs(lz[b]), 1.0), (b, objf[b], lz[b])
        assert np.abs(grad[b].astype(np.float64) - gamma[b]).max() <= GRAD_ATOL, b
        ok += 1
    return ok


def test_all_final_left_to_right_graph_without_a_leak():
    # every state final, so the old criterion (fp32 iff all states final) would have
    # run these in fp32; without a leak nothing bounds how far below the frame total
    # a state that carries posterior mass can sit
    rng = np.random.default_rng(31)
    P, B = 84, 4
    lens = np.array([300, 280, 150, 40], np.int32)
    x = rng.normal(0, 2, (B, 300, P)).astype(np.float32)
    for b in range(B):
        x[b, lens[b]:] = np.nan
    # a unique start state: fp64, every element matches
    graphs = [_left_to_right(rng, 75, P, False) for _ in range(B)]
    h = binding.lfmmi_graph_create_batch(graphs)
    assert binding.lfmmi_graph_info(h)["fp64"] == 1
    lz, gamma = oracle.forward_backward_per_utt(graphs, x, lens, 0.0)
    check(*run_gpu(h, x, lens, 0.0), lz, gamma, "all final, one start state, no leak")
    h.close()
    # every state initial as well: fp32; with the leak it is bounded and matches,
    # without it a sequence matches or comes back flagged
    graphs = [_left_to_right(rng, 75, P, True) for _ in range(B)]
    h = binding.lfmmi_graph_create_batch(graphs)
    assert binding.lfmmi_graph_info(h)["fp64"] == 0
    lz, gamma = oracle.forward_backward_per_utt(graphs, x, lens, 1e-5)
    check(*run_gpu(h, x, lens, 1e-5), lz, gamma, "all final and initial, leak")
    lz, gamma = oracle.forward_backward_per_utt(graphs, x, lens, 0.0)
    ok = _match_or_flagged(run_gpu(h, x, lens, 0.0), lz, gamma, lens)
    print("all final and initial, no leak, fp32: %d of %d sequences unflagged and matching" % (ok, B))
    h.close()


def test_forced_fp32_on_numerator_graphs_matches_or_is_flagged(monkeypatch):
    # LFMMI_PRECISION=32 overrides the choice of fp64 for left-to-right graphs; mass
    # that underflows then shows as a dead sequence or as passes that disagree
    wl = workloads.make_workload(5, scale={"S": 300, "B": 12, "nlo": 20, "nhi": 120})
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    lz, gamma = oracle.forward_backward_per_utt(wl["num"], x, lens, leak)
    monkeypatch.setenv("LFMMI_PRECISION", "32")
    h = binding.lfmmi_graph_create_batch(wl["num"])
    monkeypatch.delenv("LFMMI_PRECISION")
    assert binding.lfmmi_graph_info(h)["fp64"] == 0
    ok = _match_or_flagged(run_gpu(h, x, lens, leak), lz, gamma, lens)
    print("numerators forced to fp32: %d of %d sequences unflagged and matching" % (ok, len(lens)))
    h.close()
    h = binding.lfmmi_graph_create_batch(wl["num"])
    assert binding.lfmmi_graph_info(h)["fp64"] == 1
    check(*run_gpu(h, x, lens, leak), lz, gamma, "numerators, fp64")
    h.close()


# ---- graphs whose arcs carry the pdf-id of the state they enter: the recursion
# variant without an emission gather (alpha multiplies a row by its emission once,
# beta folds the emission into the stored vector)
def _emission_by_state(handle):
    return binding.lfmmi_graph_info(handle)["emission_by_state"]


@pytest.mark.parametrize("kind", ["uniform_pi", "nonuniform_pi", "small", "leaks"])
def test_hmm_expanded_graph_every_element(kind, monkeypatch):
    scale = {"B": 5, "Tlo": 20, "Thi": 70}
    if kind == "small":
        scale.update(phones=9, succ=4)        # 72 states: two slices, ragged
    if kind == "nonuniform_pi":
        scale.update(succ=12)                 # 1,008 states: three registers per slot fit
    wl = workloads.make_workload(6, scale=scale, pad_value=np.nan)
    g = wl["den"]
    if kind in ("small", "nonuniform_pi"):    # few slots per wave: not taken unless asked for
        monkeypatch.setenv("LFMMI_GROUPED", "2")
    if kind == "nonuniform_pi":               # per-arc leak factors and closing slots
        rng = np.random.default_rng(3)
        pi = rng.uniform(0.05, 1.0, g["num_states"])
        g["init_prob"] = (pi / pi.sum()).astype(np.float32)
        g["final_prob"] = rng.uniform(0.2, 1.0, g["num_states"]).astype(np.float32)
    h = binding.lfmmi_graph_create(g)
    assert _emission_by_state(h) == 1 and binding.lfmmi_graph_info(h)["fp64"] == 0
    info = binding.lfmmi_graph_ordering_info(h, 0, 0)
    assert info["register_slots"] >= info["max_wave_slots"]
    leaks = (0.0, 1e-5, 0.3) if kind == "leaks" else (wl["leak"],)
    for leak in leaks:
        lz, gamma = oracle.forward_backward(g, wl["logits"], wl["lengths"], leak)
        out = run_gpu(h, wl["logits"], wl["lengths"], leak)
        check(*out, lz, gamma, "hmm graph, %s, leak %g" % (kind, leak))
        for b, Tb in enumerate(wl["lengths"]):
            assert np.all(out[1][b, Tb:] == 0.0)
    h.close()
    # the same graph through the kernels that gather the emission per arc
    monkeypatch.setenv("LFMMI_GROUPED", "0")
    h0 = binding.lfmmi_graph_create(g)
    monkeypatch.delenv("LFMMI_GROUPED")
    assert _emission_by_state(h0) == 0
    lz, gamma = oracle.forward_backward(g, wl["logits"], wl["lengths"], wl["leak"])
    check(*run_gpu(h0, wl["logits"], wl["lengths"], wl["leak"]), lz, gamma, "hmm graph, per-arc gather")
    h0.close()


def test_hmm_expanded_graph_full_size_all_sequences():
    wl = workloads.make_workload(6)
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    den = binding.lfmmi_graph_create(wl["den"])
    assert _emission_by_state(den) == 1
    objf, grad, status = run_gpu(den, x, lens, leak)
    lz, gamma = oracle.forward_backward(wl["den"], x, lens, leak)
    rel, err = check(objf, grad, status, lz, gamma, "hmm_den_2k")
    print("hmm_den_2k full size: objf max rel err %.2e, grad max abs err %.2e" % (rel, err))
    den.close()


def test_numerator_graphs_through_the_emission_by_state_variant_in_fp64(monkeypatch):
    # the phone-string numerators carry the pdf-id of the entered state; a unique start
    # state makes them fp64 with per-arc leak factors. With their few slots per wave
    # the variant is slower and not taken by default: asked for here
    wl = workloads.make_workload(5, scale={"S": 300, "B": 9, "nlo": 5, "nhi": 110})
    x, lens, leak = wl["logits"], wl["lengths"], wl["leak"]
    num = binding.lfmmi_graph_create_batch(wl["num"])
    assert binding.lfmmi_graph_info(num)["emission_by_state"] == 0
    num.close()
    monkeypatch.setenv("LFMMI_GROUPED", "2")
    num = binding.lfmmi_graph_create_batch(wl["num"])
    monkeypatch.delenv("LFMMI_GROUPED")
    info = binding.lfmmi_graph_info(num)
    assert info["fp64"] == 1 and info["emission_by_state"] == 1
    for lk in (leak, 0.0, 0.05):
        lz, gamma = oracle.forward_backward_per_utt(wl["num"], x, lens, lk)
        check(*run_gpu(num, x, lens, lk), lz, gamma, "numerators, emission by state, leak %g" % lk)
    num.close()


def test_hmm_expanded_graph_very_short_sequences():
    # lengths 0, 1, 2, 3: the emission values of a row are fetched two steps ahead and
    # must stay inside the sequence; beta folds them in before its first gather
    wl = workloads.make_workload(6, scale={"B": 6, "Tlo": 4, "Thi": 9}, pad_value=np.nan)
    g = wl["den"]
    lens = np.array([0, 1, 2, 3, 9, 4], np.int32)
    x = np.random.default_rng(8).normal(0, 2, (6, 9, g["num_pdfs"])).astype(np.float32)
    for b in range(6):
        x[b, lens[b]:] = np.nan
    h = binding.lfmmi_graph_create(g)
    assert _emission_by_state(h) == 1
    for leak in (1e-5, 0.2):
        lz, gamma = oracle.forward_backward(g, x, lens, leak)
        objf, grad, status = run_gpu(h, x, lens, leak)
        # the empty sequence: log Z = log(1 + leak), next to 0 with the default leak, where
        # the fp32 sum of the 2,016 initial probabilities decides the relative error
        assert abs(float(objf[0]) - lz[0]) <= 1e-6 and np.all(grad[0] == 0.0) and status[0] == 0
        check(objf[1:], grad[1:], status[1:], lz[1:], gamma[1:],
              "hmm graph, short sequences, leak %g" % leak)
    h.close()


def test_paper_sized_denominator_full_size_all_sequences():
    # 7,398 states and 128 sequences, the sizes of the paper's own run (Section 4.4):
    # 7,424 padded rows in the 32 KB state vectors, part of every wave's arcs streamed
    wl = _full_size(7, list(range(128)))
    assert wl["den"]["num_states"] * 128 == 946944
