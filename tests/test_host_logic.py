"""CPU-side tests: the C-ABI library loads and exports what include/lfmmi.h
declares, the graph packer keeps every arc exactly once in each of its three
orderings, and argument errors come back as status codes with a message.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2005_09824_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lfmmi.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)  # declarations only
    declared = set(re.findall(r"\b(lfmmi_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = binding.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


def _unpack(graph_handle, g, graph):
    """Rebuild (src, dst, pdf, w) lists from each packed ordering."""
    od = [binding.lfmmi_graph_ordering_copy(graph_handle, g, o) for o in range(3)]
    state_of = [od[0]["row_id"], od[1]["row_id"]]  # position -> state, per numbering
    out = []
    for o in range(3):
        d = od[o]
        arcs = []
        assert d["slice_off"][0] == 0 and d["slice_off"][-1] == d["total_slots"]
        assert d["wave_first"][0] == 0 and d["wave_first"][-1] == d["slices"]
        assert np.all(np.diff(d["wave_first"]) >= 0)
        per_wave = []
        for wv in range(d["waves"]):
            s0, s1 = d["wave_first"][wv], d["wave_first"][wv + 1]
            per_wave.append(int(d["slice_off"][s1] - d["slice_off"][s0]))
        assert max(per_wave) == d["max_wave_slots"]
        for s in range(d["slices"]):
            o0, o1 = d["slice_off"][s], d["slice_off"][s + 1]
            if o < 2 and d["closing_slots"]:   # it carries the row's leak-dot weight
                o1 -= 1
                for lane in range(64):
                    row = s * 64 + lane
                    st = d["row_id"][row]
                    want = 0.0 if st < 0 else (1.0 if o == 0 else float(graph["init_prob"][st]))
                    assert d["key"][o1 * 64 + lane] == 0
                    assert d["w"][o1 * 64 + lane] == np.float32(want)
            hub = o < 2 and d["slice_hub"][s]
            if hub:  # all 64 lanes hold arcs of lane 0's row; the other rows are padding
                assert d["row_id"][s * 64] >= 0 and np.all(d["row_id"][s * 64 + 1:s * 64 + 64] < 0)
            for lane in range(64):
                row = s * 64 if hub else s * 64 + lane
                for i in range(o0, o1):
                    k, w = int(d["key"][i * 64 + lane]), float(d["w"][i * 64 + lane])
                    if w == 0.0:      # padding: anywhere in the row (slots are ordered to
                        continue      # spread LDS banks); its key points at an unused bank
                    assert d["row_id"][row] >= 0
                    x, y = (k & 0xFFFF) // 4, (k >> 16) // 4
                    if o == 0:
                        arcs.append((int(state_of[0][x]), int(d["row_id"][row]), y, w))
                    elif o == 1:
                        arcs.append((int(d["row_id"][row]), int(state_of[1][x]), y, w))
                    else:
                        arcs.append((int(state_of[0][x]), int(state_of[1][y]),
                                     int(d["row_id"][row]), w))
        out.append(sorted(arcs))
    want = sorted(zip(graph["src"].tolist(), graph["dst"].tolist(), graph["pdf"].tolist(),
                      np.exp(graph["logw"].astype(np.float64)).astype(np.float32).tolist()))
    return out, want, od


@pytest.mark.parametrize("which", ["tiny", "den_scaled", "zipf"])
def test_pack_keeps_every_arc_once(which):
    if which == "tiny":
        g = workloads.make_workload(1)["den"]
    elif which == "den_scaled":
        g = workloads.make_workload(2, scale={"S": 300, "B": 2, "Tlo": 5, "Thi": 6})["den"]
    else:
        g = workloads.make_workload(3, scale={"S": 200, "P": 50, "B": 2, "Tlo": 5, "Thi": 6})["den"]
    h = binding.lfmmi_graph_pack(g)
    got, want, od = _unpack(h, 0, g)
    for o in range(3):
        assert got[o] == want, "ordering %d lost or changed arcs" % o
    S = g["num_states"]
    for o in range(2):
        ids = od[o]["row_id"]
        assert sorted(ids[ids >= 0].tolist()) == list(range(S))  # a permutation of the states
        assert od[o]["rows"] == S and od[o]["slices"] == (S + 63) // 64
    info = binding.lfmmi_graph_info(h)
    assert info["num_graphs"] == 1 and info["total_arcs"] == len(g["src"]) and info["uploaded"] == 0
    h.close()


def test_pack_batch_of_numerators():
    wl = workloads.make_workload(5, scale={"B": 5, "nlo": 3, "nhi": 9})
    h = binding.lfmmi_graph_pack_batch(wl["num"])
    assert binding.lfmmi_graph_info(h)["num_graphs"] == 5
    for g in range(5):
        got, want, _ = _unpack(h, g, wl["num"][g])
        for o in range(3):
            assert got[o] == want
    h.close()


def test_pack_waves_are_balanced():
    g = workloads.make_workload(2)["den"]
    h = binding.lfmmi_graph_pack(g)
    info = binding.lfmmi_graph_info(h)
    assert info["rec_waves"] == 16
    for o in range(3):
        oi = binding.lfmmi_graph_ordering_info(h, 0, o)
        ideal = len(g["src"]) / (64.0 * oi["waves"])
        assert oi["max_wave_slots"] <= 1.35 * ideal + 4, (o, oi, ideal)
    h.close()


def test_slot_ordering_lowers_modelled_bank_conflicts(monkeypatch):
    g = workloads.make_workload(2)["den"]
    tuned = binding.lfmmi_graph_pack(g)
    monkeypatch.setenv("LFMMI_BALANCE", "0")
    monkeypatch.setenv("LFMMI_ORDER", "0")
    plain = binding.lfmmi_graph_pack(g)
    for o in range(3):
        a = binding.lfmmi_graph_ordering_info(tuned, 0, o)
        b = binding.lfmmi_graph_ordering_info(plain, 0, o)
        floor = 2 * a["total_slots"] * (1 if o < 2 else 2)  # one cycle per half-wave gather
        assert floor <= a["gather_cycles"] <= 0.7 * b["gather_cycles"], (o, a, b)
    tuned.close(); plain.close()


@pytest.mark.parametrize("which", ["den", "hmm"])
def test_occupancy_arcs_dealt_to_rows_and_slots_keep_every_arc(which, monkeypatch):
    # the occupancy ordering may place an arc in any row of its pdf: both placements hold every
    # arc once, in a row of its pdf, and the one that is kept is never the dearer of the two
    if which == "den":
        g = workloads.make_workload(2, scale={"B": 2, "Tlo": 5, "Thi": 6})["den"]
    else:
        g = workloads.make_workload(6, scale={"B": 2, "Tlo": 5, "Thi": 6})["den"]
    both = binding.lfmmi_graph_pack(g)
    monkeypatch.setenv("LFMMI_DEAL", "0")
    ordered = binding.lfmmi_graph_pack(g)
    for h in (both, ordered):
        got, want, _ = _unpack(h, 0, g)
        assert got[2] == want
    a = binding.lfmmi_graph_ordering_info(both, 0, 2)
    b = binding.lfmmi_graph_ordering_info(ordered, 0, 2)
    assert a["total_slots"] == b["total_slots"] and a["rows"] == b["rows"]
    assert 4 * a["total_slots"] <= a["gather_cycles"] <= b["gather_cycles"]
    if which == "den":  # random pdfs on the arcs: the joint placement wins
        assert a["gather_cycles"] <= 0.95 * b["gather_cycles"], (a, b)
    both.close(); ordered.close()


def test_graph_with_no_arcs_and_isolated_states():
    g = {"num_states": 3, "num_pdfs": 2, "src": np.zeros(0, np.int32), "dst": np.zeros(0, np.int32),
         "pdf": np.zeros(0, np.int32), "logw": np.zeros(0, np.float32),
         "init_prob": np.ones(3, np.float32), "final_prob": np.ones(3, np.float32)}
    h = binding.lfmmi_graph_pack(g)
    assert binding.lfmmi_graph_ordering_info(h, 0, 0)["total_slots"] == 2  # uniform pi: no closing slot, two padding slots
    assert binding.lfmmi_graph_ordering_info(h, 0, 2)["total_slots"] == 0  # no rows at all
    h.close()


def _tiny():
    return {"num_states": 2, "num_pdfs": 2, "src": np.array([0, 1], np.int32),
            "dst": np.array([1, 0], np.int32), "pdf": np.array([0, 1], np.int32),
            "logw": np.zeros(2, np.float32), "init_prob": np.array([1, 0], np.float32),
            "final_prob": np.array([0, 1], np.float32)}


@pytest.mark.parametrize("field,value,code", [
    ("src", np.array([0, 2], np.int32), 2),
    ("dst", np.array([-1, 0], np.int32), 2),
    ("pdf", np.array([0, 2], np.int32), 2),
    ("logw", np.array([0, np.nan], np.float32), 2),
    ("logw", np.array([-np.inf, 0], np.float32), 2),
    ("init_prob", np.array([-1, 0], np.float32), 2),
    ("final_prob", np.array([np.inf, 0], np.float32), 2),
])
def test_bad_graphs_are_refused(field, value, code):
    g = _tiny()
    g[field] = value
    with pytest.raises(binding.LfmmiError) as ei:
        binding.lfmmi_graph_pack(g)
    assert ei.value.code == code and str(ei.value)


def test_unsupported_sizes_and_invalid_arguments():
    g = _tiny()
    g["num_pdfs"] = 20000
    with pytest.raises(binding.LfmmiError) as ei:
        binding.lfmmi_graph_pack(g)
    assert ei.value.code == 5
    big = {"num_states": 17000, "num_pdfs": 2, "src": np.zeros(1, np.int32),
           "dst": np.zeros(1, np.int32), "pdf": np.zeros(1, np.int32),
           "logw": np.zeros(1, np.float32), "init_prob": np.ones(17000, np.float32),
           "final_prob": np.ones(17000, np.float32)}
    with pytest.raises(binding.LfmmiError) as ei:
        binding.lfmmi_graph_pack(big)
    assert ei.value.code == 5
    lib = binding.load_library()
    out = ctypes.c_void_p()
    assert lib.lfmmi_graph_pack(0, 1, 0, None, None, None, None, None, None, ctypes.byref(out)) == 1
    assert lib.lfmmi_graph_pack(1, 1, 0, None, None, None, None, None, None, ctypes.byref(out)) == 1
    assert "null" in binding.lfmmi_last_error()
    assert lib.lfmmi_forward_backward(None, None, None, 1, 1, 1, 0.0, 1.0, 0, None, None, None, None) == 1
    # a packed-only handle cannot run
    h = binding.lfmmi_graph_pack(_tiny())
    lens = np.array([1], np.int32)
    rc = lib.lfmmi_forward_backward(h.handle, None, ctypes.c_void_p(lens.ctypes.data), 1, 1, 2,
                                    0.0, 1.0, 0, None, None, None, None)
    assert rc == 1 and "not uploaded" in binding.lfmmi_last_error()
    h.close()
    lib.lfmmi_graph_destroy(None)  # no-op


def test_fst_text_reader_round_trip_and_errors():
    from paper_2005_09824_amd import fst_text
    text = """0 1 3 3 0.5
1 1 3 3 0.25
1 2 5 5
2 0.125
"""
    g = fst_text.read_fst_text(text.splitlines())
    assert g["num_states"] == 3 and g["num_pdfs"] == 5
    assert g["src"].tolist() == [0, 1, 1] and g["dst"].tolist() == [1, 1, 2]
    assert g["pdf"].tolist() == [2, 2, 4]
    assert np.allclose(g["logw"], [-0.5, -0.25, 0.0])
    assert g["init_prob"].tolist() == [1.0, 0.0, 0.0]
    assert np.allclose(g["final_prob"], [0.0, 0.0, np.exp(-0.125)])
    # acceptor columns, explicit pdf count, another start state
    g2 = fst_text.read_fst_text(["4 2 1 0.5", "2 2 2", "2"], num_pdfs=7, acceptor=True)
    assert g2["num_states"] == 5 and g2["num_pdfs"] == 7 and g2["init_prob"][4] == 1.0
    assert g2["final_prob"][2] == 1.0 and g2["pdf"].tolist() == [0, 1]
    # what it writes it reads back
    back = fst_text.read_fst_text(fst_text.write_fst_text(g))
    for k in ("src", "dst", "pdf"):
        assert back[k].tolist() == g[k].tolist()
    assert np.allclose(back["logw"], g["logw"]) and np.allclose(back["final_prob"], g["final_prob"])
    # the packer accepts it
    h = binding.lfmmi_graph_pack(g)
    assert binding.lfmmi_graph_info(h)["total_arcs"] == 3
    h.close()
    for bad in (["0 1 0 0 1.0"], ["0 1 x 1"], ["0 1 2 2 inf"], ["3"], ["0 1 2 2 0.1 9"]):
        with pytest.raises(ValueError):
            fst_text.read_fst_text(bad)
    with pytest.raises(ValueError):
        fst_text.read_fst_text(["0 1 9 9"], num_pdfs=4)


def _hub_graph(seed=5, S=500, in_hub=300, out_hub=200):
    rng = np.random.default_rng(seed)
    g = workloads.random_den_graph(rng, S, 8, 30, 0.5)
    extra_src = rng.choice(S, size=in_hub, replace=False).astype(np.int32)       # into state 7
    extra_dst = rng.choice(S, size=out_hub, replace=False).astype(np.int32)      # out of state 11
    g["src"] = np.concatenate([g["src"], extra_src, np.full(out_hub, 11, np.int32)])
    g["dst"] = np.concatenate([g["dst"], np.full(in_hub, 7, np.int32), extra_dst])
    n = in_hub + out_hub
    g["pdf"] = np.concatenate([g["pdf"], rng.integers(0, 30, n).astype(np.int32)])
    g["logw"] = np.concatenate([g["logw"], np.log(rng.uniform(0.01, 0.2, n)).astype(np.float32)])
    return g


@pytest.mark.parametrize("nonuniform", [False, True])
def test_hub_states_get_slices_of_their_own(nonuniform):
    g = _hub_graph()
    if nonuniform:  # closing slots: the hub's leak-dot weight sits in lane 0 only
        pi = np.random.default_rng(1).uniform(0.1, 1.0, g["num_states"])
        g["init_prob"] = (pi / pi.sum()).astype(np.float32)
    h = binding.lfmmi_graph_pack(g)
    got, want, od = _unpack(h, 0, g)
    for o in range(3):
        assert got[o] == want, "ordering %d lost or changed arcs" % o
    # one hub slice per direction, a few slots wide instead of hundreds
    for o, (state, deg) in enumerate(((7, 300), (11, 200))):
        assert od[o]["hub_slices"] == 1
        s = int(np.flatnonzero(od[o]["slice_hub"])[0])
        assert od[o]["row_id"][s * 64] == state
        width = od[o]["slice_off"][s + 1] - od[o]["slice_off"][s]
        assert width <= (deg + 10 + 63) // 64 + 3 and width % 2 == 0
        assert od[o]["max_wave_slots"] < 64
    assert od[2]["hub_slices"] == 0
    h.close()


def _many_hubs(S, hubs_in, hubs_out, deg=600, seed=9, k=9, P=84):
    """Random graph plus `hubs_in` states with `deg` arcs into them and `hubs_out`
    states with `deg` arcs out of them."""
    rng = np.random.default_rng(seed)
    g = workloads.random_den_graph(rng, S, k, P, 0.5)
    src, dst = [g["src"]], [g["dst"]]
    for h in range(hubs_in):
        src.append(rng.choice(S, size=deg, replace=False).astype(np.int32))
        dst.append(np.full(deg, 10 + h, np.int32))
    for h in range(hubs_out):
        src.append(np.full(deg, 5000 % S + h, np.int32))
        dst.append(rng.choice(S, size=deg, replace=False).astype(np.int32))
    n = (hubs_in + hubs_out) * deg
    g["src"], g["dst"] = np.concatenate(src), np.concatenate(dst)
    g["pdf"] = np.concatenate([g["pdf"], rng.integers(0, P, n).astype(np.int32)])
    g["logw"] = np.concatenate([g["logw"], np.log(rng.uniform(0.001, 0.01, n)).astype(np.float32)])
    return g


@pytest.mark.parametrize("S,hubs_in,hubs_out", [
    (8000, 8, 0),     # 8000 states fit a 32 KB state vector, 8512 padded rows do not
    (8000, 20, 3),
    (12200, 0, 4),    # ... nor do 12288 + 3 * 64 the 48 KB map (P > 255: plain emission rows)
    (4000, 6, 6),     # fits: the register / hybrid kernels stay
])
def test_padded_rows_of_hub_slices_fit_the_chosen_kernels_lds_map(S, hubs_in, hubs_out):
    # every hub state gets a slice of its own, i.e. 63 padding rows: what must fit
    # the fixed LDS map of the register-resident kernels is the padded row count
    g = _many_hubs(S, hubs_in, hubs_out, P=300 if S > 12000 else 84)
    h = binding.lfmmi_graph_pack(g)
    for o in (0, 1):
        info = binding.lfmmi_graph_ordering_info(h, 0, o)
        assert info["hub_slices"] == (hubs_in, hubs_out)[o]
        assert info["slices"] * 64 >= S + 63 * info["hub_slices"]
        if info["register_slots"] > 0:
            assert info["slices"] * 64 <= info["lds_vector_rows"], info
        else:
            assert info["lds_vector_rows"] == 0
    rows = max(binding.lfmmi_graph_ordering_info(h, 0, o)["slices"] * 64 for o in (0, 1))
    resident = binding.lfmmi_graph_ordering_info(h, 0, 0)["register_slots"] > 0
    if S == 4000:
        assert resident and rows <= 8192
    elif S == 8000:   # the map with 48 KB state vectors (plain emission rows), or streamed arcs
        assert rows > 8192
        assert not resident or binding.lfmmi_graph_ordering_info(h, 0, 0)["lds_vector_rows"] == 12288
    else:
        assert rows > 12288 and not resident
    h.close()


def test_hub_slices_are_given_up_when_their_padding_rows_overflow_the_key_fields():
    # 16300 states and 5 out-degree hubs: 16640 BWD rows would not fit the 16-bit
    # (row * 4) fields of the arc records; the graph is packed without hub slices
    g = _many_hubs(16300, 0, 5, deg=300, k=2, P=40)
    h = binding.lfmmi_graph_pack(g)
    got, want, od = _unpack(h, 0, g)
    for o in range(3):
        assert got[o] == want, "ordering %d lost or changed arcs" % o
        assert od[o]["hub_slices"] == 0
    for o in (0, 1):
        assert od[o]["slices"] * 64 <= 16384
        assert int((od[o]["key"] & 0xFFFF).max()) // 4 < od[o]["slices"] * 64
    # OCC keys: both fields are row numbers
    assert int((od[2]["key"] >> 16).max()) // 4 < od[1]["slices"] * 64
    h.close()


def test_packer_finds_graphs_whose_pdf_is_a_function_of_the_entered_state(monkeypatch):
    wl6 = workloads.make_workload(6, scale={"B": 2, "Tlo": 3, "Thi": 4})
    g = wl6["den"]
    pdf_of = {}
    for d, p in zip(g["dst"].tolist(), g["pdf"].tolist()):
        assert pdf_of.setdefault(d, p) == p       # the generator's own promise
    h = binding.lfmmi_graph_pack(g)
    assert binding.lfmmi_graph_info(h)["emission_by_state"] == 1
    h.close()
    g2 = dict(g)
    pdf = g["pdf"].copy()
    pdf[5] = (pdf[5] + 1) % g["num_pdfs"]         # one arc breaks it
    g2["pdf"] = pdf
    h = binding.lfmmi_graph_pack(g2)
    assert binding.lfmmi_graph_info(h)["emission_by_state"] == 0
    h.close()
    # random pdf-ids per arc (the five named workloads' denominators): never
    h = binding.lfmmi_graph_pack(workloads.make_workload(2, scale={"S": 200, "B": 2})["den"])
    assert binding.lfmmi_graph_info(h)["emission_by_state"] == 0
    h.close()
    # phone-string numerators: yes (when asked for: with their few slots per wave the
    # variant does not pay); a batch with one graph that is not: no
    monkeypatch.setenv("LFMMI_GROUPED", "2")
    wl5 = workloads.make_workload(5, scale={"S": 100, "B": 3, "nlo": 3, "nhi": 6})
    h = binding.lfmmi_graph_pack_batch(wl5["num"])
    assert binding.lfmmi_graph_info(h)["emission_by_state"] == 1
    h.close()
    mixed = list(wl5["num"])
    bad = dict(mixed[1])
    bad["pdf"] = (mixed[1]["pdf"] + np.arange(len(mixed[1]["pdf"]))) % 84
    mixed[1] = bad
    h = binding.lfmmi_graph_pack_batch(mixed)
    assert binding.lfmmi_graph_info(h)["emission_by_state"] == 0
    h.close()


def test_bench_refuses_more_than_one_gpu():
    # one GPU is the whole target: the command says so and exits before it touches a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
