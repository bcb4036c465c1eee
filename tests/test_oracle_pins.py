"""Pins for the fp64 CPU oracle: closed forms, brute force, a dense twin,
invariants, finite differences and the paper's printed worked examples.
Each pin is chosen so that a plausible slip (dropped leak application, wrong
time index, transposed arc, pdf mix-up, missing final probability) fails it.
"""
import math
import os

import numpy as np
import pytest

from oracle import lfmmi_oracle as oracle
from paper_2005_09824_amd import workloads
from tests import pins

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def fb(graph, x, leak, lengths=None, **kw):
    x = np.asarray(x, dtype=np.float32)
    if x.ndim == 2:
        x = x[None]
    if lengths is None:
        lengths = np.full(x.shape[0], x.shape[1], dtype=np.int32)
    return oracle.forward_backward(graph, x, np.asarray(lengths, np.int32), leak, **kw)


# ---- P1: one state, closed form (pins leak count/placement and time indexing)
@pytest.mark.parametrize("T", [0, 1, 7])
@pytest.mark.parametrize("eps", [0.0, 1e-5, 0.3])
def test_p1_single_state_closed_form(T, eps):
    rng = np.random.default_rng(1)
    w = 0.7
    g = pins.small_graph(1, 1, [(0, 0, 0, w)], [1.0], [1.0])
    x = rng.normal(size=(1, max(T, 1), 1)).astype(np.float32)
    logz, gamma = fb(g, x, eps, lengths=[T])
    lw = float(np.float32(np.log(w)))  # the weight as the oracle sees it (fp32 log)
    want = T * lw + float(x[0, :T, 0].astype(np.float64).sum()) + (T + 1) * math.log1p(eps)
    assert abs(logz[0] - want) < 1e-12 * max(1.0, abs(want))
    assert np.allclose(gamma[0, :T, 0], 1.0, atol=1e-12)


# ---- P2: stochastic graph, frame-constant logits (any topology)
@pytest.mark.parametrize("eps", [0.0, 1e-5, 0.05])
def test_p2_stochastic_graph_closed_form(eps):
    rng = np.random.default_rng(2)
    g = workloads.random_den_graph(rng, 50, 4, 7, 0.5)
    # make the fp32 log-weights exactly stochastic in fp64 by renormalising what
    # the oracle will see: w = exp(float32 logw); scale tolerance covers the rest
    T = 12
    c = rng.normal(size=T)
    x = np.repeat(c[:, None], 7, axis=1).astype(np.float32)
    logz, gamma = fb(g, x, eps)
    w = np.exp(g["logw"].astype(np.float64)).reshape(50, 5)
    assert np.allclose(w.sum(1), 1.0, atol=1e-6)
    want = float(x[:, 0].astype(np.float64).sum()) + (T + 1) * math.log1p(eps)
    assert abs(logz[0] - want) < 1e-5  # limited by fp32 rounding of the weights
    assert np.allclose(gamma[0].sum(1), 1.0, atol=1e-12)


# ---- P3: single path (arc / pdf / time alignment, final probability)
def test_p3_single_path():
    rng = np.random.default_rng(3)
    K, P = 6, 4
    pdfs = [3, 0, 2, 2, 1]
    ws = [0.9, 0.5, 0.25, 0.7, 0.3]
    arcs = [(i, i + 1, pdfs[i], ws[i]) for i in range(K - 1)]
    init = np.zeros(K); init[0] = 1.0
    fin = np.zeros(K); fin[K - 1] = 0.6
    g = pins.small_graph(K, P, arcs, init, fin)
    x = rng.normal(size=(K - 1, P)).astype(np.float32)
    logz, gamma = fb(g, x, 0.0)
    want = sum(float(np.float32(np.log(ws[t]))) + float(x[t, pdfs[t]]) for t in range(K - 1))
    want += math.log(float(np.float32(0.6)))
    assert abs(logz[0] - want) < 1e-12
    expect = np.zeros((K - 1, P))
    for t in range(K - 1):
        expect[t, pdfs[t]] = 1.0
    assert np.allclose(gamma[0], expect, atol=1e-12)
    # one frame too many or too few: no path reaches the final state
    for T in (K - 2, K):
        xx = rng.normal(size=(T, P)).astype(np.float32)
        lz, gm = fb(g, xx, 0.0)
        assert lz[0] == -np.inf and np.all(gm == 0.0)


# ---- P4: counting paths through a chain with self-loops
@pytest.mark.parametrize("K,T", [(3, 5), (4, 9), (8, 30)])
def test_p4_chain_counting(K, T):
    arcs = []
    for i in range(K):
        arcs.append((i, i, 0, 1.0))
        if i + 1 < K:
            arcs.append((i, i + 1, 0, 1.0))
    init = np.zeros(K); init[0] = 1.0
    fin = np.zeros(K); fin[K - 1] = 1.0
    g = pins.small_graph(K, 1, arcs, init, fin)
    x = np.zeros((T, 1), dtype=np.float32)
    logz, _ = fb(g, x, 0.0)
    assert abs(logz[0] - math.log(math.comb(T, K - 1))) < 1e-11


# ---- P5: brute-force path enumeration, leak as an explicit path choice
@pytest.mark.parametrize("seed", range(6))
def test_p5_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    S = int(rng.integers(2, 4))
    P = int(rng.integers(1, 4))
    T = int(rng.integers(1, 5))
    eps = [0.0, 1e-5, 0.2][seed % 3]
    g = pins.random_small_graph(rng, S, P, n_arcs=int(rng.integers(S, 3 * S)),
                                one_hot_init=(seed % 2 == 0),
                                sparse_final=(seed % 2 == 1))
    x = rng.normal(size=(T, P)).astype(np.float32)
    Z, gam = pins.brute_force(g, x, eps)
    logz, gamma = fb(g, x, eps)
    if Z == 0:
        assert logz[0] == -np.inf
    else:
        assert abs(logz[0] - math.log(Z)) < 1e-12 * max(1, abs(math.log(Z)))
        assert np.allclose(gamma[0], gam, atol=1e-12)


# ---- P6: dense probability-domain twin on config 1 (den and both numerators)
def test_p6_dense_twin_config1():
    wl = workloads.make_workload(1)
    graphs = [wl["den"], wl["den"]], wl["num"]
    for glist in graphs:
        for b in range(2):
            T = int(wl["lengths"][b])
            x = wl["logits"][b, :T]
            Z, gam, Zb = pins.dense_twin(glist[b], x, wl["leak"])
            logz, gamma, logz_b = fb(glist[b], x, wl["leak"], return_bwd_total=True)
            assert abs(logz[0] - math.log(Z)) < 1e-10
            assert abs(logz_b[0] - math.log(Zb)) < 1e-10
            assert np.allclose(gamma[0], gam, atol=1e-11)


def test_p6_dense_twin_large_leak_general_pi():
    rng = np.random.default_rng(66)
    g = pins.random_small_graph(rng, 7, 5, 25)
    x = rng.normal(size=(9, 5)).astype(np.float32)
    Z, gam, Zb = pins.dense_twin(g, x, 0.37)
    logz, gamma, logz_b = fb(g, x, 0.37, return_bwd_total=True)
    assert abs(logz[0] - math.log(Z)) < 1e-11
    assert abs(logz_b[0] - math.log(Zb)) < 1e-11
    assert np.allclose(gamma[0], gam, atol=1e-12)


# ---- P7: invariants
def _case(seed=7, S=30, k=3, P=6, B=3, T=14):
    rng = np.random.default_rng(seed)
    g = workloads.random_den_graph(rng, S, k, P, 0.5)
    g["init_prob"] = rng.uniform(0.0, 1.0, S).astype(np.float32)
    g["final_prob"] = rng.uniform(0.0, 1.0, S).astype(np.float32)
    lengths = np.asarray([T, T - 3, T - 7], dtype=np.int32)[:B]
    x = workloads.random_logits(rng, lengths, P, 2.0)
    return g, x, lengths


def test_p7_forward_backward_totals_and_row_sums():
    g, x, lengths = _case()
    logz, gamma, logz_b = oracle.forward_backward(g, x, lengths, 1e-3,
                                                  return_bwd_total=True)
    assert np.allclose(logz, logz_b, atol=1e-11)
    for b, Tb in enumerate(lengths):
        assert np.all(gamma[b] >= 0)
        assert np.allclose(gamma[b, :Tb].sum(1), 1.0, atol=1e-12)
        assert np.all(gamma[b, Tb:] == 0.0)


def test_p7_padding_is_never_read():
    g, x, lengths = _case()
    ref = oracle.forward_backward(g, x, lengths, 1e-3)
    x2 = x.copy()
    for b, Tb in enumerate(lengths):
        x2[b, Tb:] = np.nan
    got = oracle.forward_backward(g, x2, lengths, 1e-3)
    assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])
    # and a sequence alone gives what it gives inside the batch
    for b, Tb in enumerate(lengths):
        lz, gm = oracle.forward_backward(g, x[b:b + 1, :Tb], lengths[b:b + 1], 1e-3)
        assert lz[0] == ref[0][b] and np.array_equal(gm[0], ref[1][b, :Tb])


def test_p7_shift_and_weight_scaling():
    g, x, lengths = _case(B=1)
    T = int(lengths[0])
    lz0, gm0 = oracle.forward_backward(g, x, lengths, 1e-4)
    c = np.float32(0.5)  # exactly representable shift of one frame
    x1 = x.copy(); x1[0, 4, :] += c
    lz1, gm1 = oracle.forward_backward(g, x1, lengths, 1e-4)
    assert abs(lz1[0] - lz0[0] - 0.5) < 1e-5  # fp32 rounding of x + c
    assert np.allclose(gm1, gm0, atol=1e-6)
    g2 = dict(g); g2["logw"] = (g["logw"].astype(np.float64) + math.log(2.0)).astype(np.float32)
    d = float(np.mean(g2["logw"].astype(np.float64) - g["logw"].astype(np.float64)))
    lz2, gm2 = oracle.forward_backward(g2, x, lengths, 1e-4)
    assert abs(lz2[0] - lz0[0] - T * d) < 1e-4
    assert np.allclose(gm2, gm0, atol=1e-6)


def test_p7_relabelling_arc_order_batch_permutation():
    g, x, lengths = _case()
    rng = np.random.default_rng(70)
    S = g["num_states"]
    ref = oracle.forward_backward(g, x, lengths, 1e-3)
    perm = rng.permutation(S)          # new label of old state s is perm[s]
    order = rng.permutation(len(g["src"]))
    g2 = dict(g)
    g2["src"] = perm[g["src"]][order].astype(np.int32)
    g2["dst"] = perm[g["dst"]][order].astype(np.int32)
    g2["pdf"] = g["pdf"][order]
    g2["logw"] = g["logw"][order]
    ip = np.empty(S, np.float32); ip[perm] = g["init_prob"]; g2["init_prob"] = ip
    fp = np.empty(S, np.float32); fp[perm] = g["final_prob"]; g2["final_prob"] = fp
    got = oracle.forward_backward(g2, x, lengths, 1e-3)
    assert np.allclose(ref[0], got[0], atol=1e-11)
    assert np.allclose(ref[1], got[1], atol=1e-12)
    bp = np.asarray([2, 0, 1])
    got = oracle.forward_backward(g, x[bp], lengths[bp], 1e-3)
    assert np.array_equal(ref[0][bp], got[0]) and np.array_equal(ref[1][bp], got[1])


def test_p7_leak_zero_is_plain_hmm_and_continuous():
    g, x, lengths = _case(B=1)
    T = int(lengths[0])
    Z, gam, _ = pins.dense_twin(g, x[0, :T], 0.0)
    lz0, gm0 = oracle.forward_backward(g, x, lengths, 0.0)
    assert abs(lz0[0] - math.log(Z)) < 1e-11 and np.allclose(gm0[0, :T], gam, atol=1e-12)
    lz1, gm1 = oracle.forward_backward(g, x, lengths, 1e-12)
    assert abs(lz1[0] - lz0[0]) < 1e-8 and np.allclose(gm1, gm0, atol=1e-8)


def test_p7_leak_revives_dead_ends():
    # chain too long for T: dead without the leak, alive with it
    K, T = 6, 3
    arcs = [(i, i + 1, 0, 1.0) for i in range(K - 1)] + [(K - 1, K - 1, 0, 1.0)]
    init = np.zeros(K); init[0] = 1.0
    fin = np.zeros(K); fin[0] = 1.0   # only the start state is final
    g = pins.small_graph(K, 1, arcs, init, fin)
    x = np.zeros((T, 1), dtype=np.float32)
    lz, _ = fb(g, x, 0.0)
    assert lz[0] == -np.inf
    eps = 0.01
    Z, gam, _ = pins.dense_twin(g, x, eps)
    lz, gm = fb(g, x, eps)
    assert Z > 0 and abs(lz[0] - math.log(Z)) < 1e-12
    assert np.allclose(gm[0], gam, atol=1e-12)


# ---- P8: the gradient is the derivative of the objective (leak terms included)
def _fd_check(graph, x, lengths, leak, entries, num=None):
    h = np.float32(2.0 ** -10)
    x = (np.round(x.astype(np.float64) * 1024) / 1024).astype(np.float32)

    def objective(xx):
        lz, _ = oracle.forward_backward(graph, xx, lengths, leak, want_gamma=False)
        return lz

    _, gamma = oracle.forward_backward(graph, x, lengths, leak)
    worst = 0.0
    for (b, t, d) in entries:
        def D(step):
            xp = x.copy(); xp[b, t, d] += step
            xm = x.copy(); xm[b, t, d] -= step
            return (objective(xp)[b] - objective(xm)[b]) / (2.0 * float(step))
        fd = (4.0 * D(h) - D(2 * h)) / 3.0   # Richardson: O(h^4)
        worst = max(worst, abs(fd - gamma[b, t, d]))
    return worst


def test_p8_finite_differences_config1_all_entries():
    wl = workloads.make_workload(1)
    B, T, P = wl["logits"].shape
    entries = [(b, t, d) for b in range(B) for t in range(int(wl["lengths"][b]))
               for d in range(P)]
    assert _fd_check(wl["den"], wl["logits"], wl["lengths"], wl["leak"], entries) < 2e-8
    # a large leak makes the leak terms of the derivative visible
    assert _fd_check(wl["den"], wl["logits"], wl["lengths"], 0.2, entries[::7]) < 2e-8
    for b in range(B):
        ent = [(0, t, d) for t in range(0, int(wl["lengths"][b]), 3) for d in range(P)]
        assert _fd_check(wl["num"][b], wl["logits"][b:b + 1], wl["lengths"][b:b + 1],
                         wl["leak"], ent) < 2e-8


def test_p8_finite_differences_config2_shaped_sample():
    wl = workloads.make_workload(2, scale={"S": 200, "B": 2, "Tlo": 20, "Thi": 30})
    rng = np.random.default_rng(8)
    entries = [(int(rng.integers(2)), int(rng.integers(20)), int(rng.integers(84)))
               for _ in range(25)]
    assert _fd_check(wl["den"], wl["logits"], wl["lengths"], wl["leak"], entries) < 2e-8


# ---- the paper's printed worked examples
def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            if line.startswith("#") or ":" not in line:
                continue
            k, v = line.split(":", 1)
            out[k.strip()] = v.strip()
    return out


def test_golden_valid_batch_sizes():
    gold = _read_golden("valid_batch_sizes.txt")
    lengths = np.asarray([int(v) for v in gold["lengths"].split()], dtype=np.int32)
    want = []
    for item in gold["bv_rle"].split():
        n, v = item.split("x")
        want += [int(v)] * int(n)
    rng = np.random.default_rng(9)
    g = workloads.random_den_graph(rng, 5, 2, 3, 1.0)
    x = workloads.random_logits(rng, lengths, 3, 1.0)
    _, gamma = oracle.forward_backward(g, x, lengths, 1e-5)
    # a frame is processed for a sequence iff its occupancy row is non-zero
    bv = (gamma.sum(2) > 0.5).sum(0)
    assert bv.tolist() == want


def test_golden_concurrent_jobs():
    gold = _read_golden("concurrent_jobs.txt")
    assert int(gold["batch"]) * int(gold["states"]) == int(gold["jobs"])


# ---- Eq. 2 / Eq. 3 composition
def test_loss_is_num_minus_den():
    wl = workloads.make_workload(1)
    objf, grad, lz_n, lz_d = oracle.loss(wl["num"], wl["den"], wl["logits"],
                                         wl["lengths"], wl["leak"])
    assert np.allclose(objf, lz_n - lz_d)
    for b in range(2):
        Tb = int(wl["lengths"][b])
        assert np.allclose(grad[b, :Tb].sum(1), 0.0, atol=1e-12)  # 1 - 1 per frame
        assert np.all(grad[b, Tb:] == 0)
