"""Seeded synthetic workloads shaped like WSJ chain training (Section 4.1-4.2, 4.4).

This module only draws random numbers and lays them out as plain numpy arrays.
It contains none of the method's arithmetic (no forward-backward, no
exponentials of logits, no graph packing), so both the HIP path and the CPU
oracle may take their inputs from it without sharing any computation.

A graph is a dict of plain arrays:
    num_states, num_pdfs : int
    src, dst, pdf        : int32 [A]   arc from-state, to-state, pdf-id
    logw                 : float32 [A] natural-log arc weight
    init_prob            : float32 [S] linear initial probability
    final_prob           : float32 [S] linear final probability

A workload is a dict with keys
    name, leak, den (graph or None), num (list of graphs or None),
    logits float32 [B, T, P], lengths int32 [B].

Draw order inside one workload is fixed: denominator topology -> weights ->
pdf-ids -> lengths -> numerator graphs -> logits -> spikes.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 2005_09824

CONFIG_NAMES = {
    1: "tiny",
    2: "wsj_mono_2k",
    3: "biphone_10k",
    4: "long_unequal_5k",
    5: "e2e_num_den",
    6: "hmm_den_2k",   # not one of the five named workloads: see make_workload
    7: "wsj_den_7398",  # likewise: the paper's own denominator size and batch
}


def random_den_graph(rng, num_states, out_arcs, num_pdfs, dirichlet,
                     pdf_dist="uniform"):
    """Random denominator-like graph.

    Every state gets a self-loop plus `out_arcs` arcs to distinct other states
    drawn without replacement; the out_arcs+1 weights of a state are one
    Dirichlet(dirichlet) draw (floored at 1e-30, not renormalised). Initial
    probability is uniform and every state is final with probability 1.
    """
    S, k = int(num_states), int(out_arcs)
    if k > S - 1:
        raise ValueError("out_arcs must be <= num_states - 1")
    src = np.repeat(np.arange(S, dtype=np.int32), k + 1)
    dst = np.empty((S, k + 1), dtype=np.int32)
    for s in range(S):
        dst[s, 0] = s
        if k:
            others = rng.choice(S - 1, size=k, replace=False)
            dst[s, 1:] = others + (others >= s)
    w = rng.dirichlet(np.full(k + 1, float(dirichlet)), size=S)
    w = np.maximum(w, 1e-30)
    A = S * (k + 1)
    if pdf_dist == "uniform":
        pdf = rng.integers(0, num_pdfs, size=A)
    elif pdf_dist == "zipf":
        ranks = np.arange(1, num_pdfs + 1, dtype=np.float64)
        p = ranks ** -1.1
        p /= p.sum()
        pdf = rng.choice(num_pdfs, size=A, p=p)
    else:
        raise ValueError(pdf_dist)
    return {
        "num_states": S,
        "num_pdfs": int(num_pdfs),
        "src": src,
        "dst": dst.reshape(-1).astype(np.int32),
        "pdf": pdf.astype(np.int32),
        "logw": np.log(w.reshape(-1)).astype(np.float32),
        "init_prob": np.full(S, 1.0 / S, dtype=np.float32),
        "final_prob": np.ones(S, dtype=np.float32),
    }


def chain_num_graph(rng, num_states, num_pdfs):
    """Left-to-right chain with self-loops: arcs i->i and i->i+1, weight 0.5,
    a uniformly random pdf-id per arc, start in state 0, end in the last."""
    K = int(num_states)
    src, dst = [], []
    for i in range(K):
        src.append(i); dst.append(i)
        if i + 1 < K:
            src.append(i); dst.append(i + 1)
    A = len(src)
    init = np.zeros(K, dtype=np.float32); init[0] = 1.0
    fin = np.zeros(K, dtype=np.float32); fin[K - 1] = 1.0
    return {
        "num_states": K,
        "num_pdfs": int(num_pdfs),
        "src": np.asarray(src, dtype=np.int32),
        "dst": np.asarray(dst, dtype=np.int32),
        "pdf": rng.integers(0, num_pdfs, size=A).astype(np.int32),
        "logw": np.full(A, np.log(0.5), dtype=np.float32),
        "init_prob": init,
        "final_prob": fin,
    }


def phone_string_num_graph(phones, num_pdfs, sil_prob=0.2):
    """Numerator graph of a phone string (phone 0 is silence, never in `phones`).

    Two states (a, b) per phone position, a start state that nothing enters,
    and an optional two-state silence between consecutive phones. Every arc
    consumes one frame and carries the pdf-id of the state it enters
    (a-state of phone k: 2k, b-state: 2k+1).
    """
    n = len(phones)
    # state numbering: 0 = start; position j (0-based): a_j = 1+2j, b_j = 2+2j;
    # gap j (between j and j+1): sa_j = 1+2n+2j, sb_j = 2+2n+2j.
    def a(j): return 1 + 2 * j
    def b(j): return 2 + 2 * j
    def sa(j): return 1 + 2 * n + 2 * j
    def sb(j): return 2 + 2 * n + 2 * j
    S = 1 + 2 * n + 2 * (n - 1)
    arcs = []  # (src, dst, pdf, weight)
    def pa(j): return 2 * int(phones[j])
    def pb(j): return 2 * int(phones[j]) + 1
    arcs.append((0, a(0), pa(0), 1.0))
    for j in range(n):
        arcs.append((a(j), a(j), pa(j), 0.5))
        arcs.append((a(j), b(j), pb(j), 0.5))
        arcs.append((b(j), b(j), pb(j), 0.5))
        if j + 1 < n:
            arcs.append((b(j), a(j + 1), pa(j + 1), 0.5 * (1.0 - sil_prob)))
            arcs.append((b(j), sa(j), 0, 0.5 * sil_prob))
            arcs.append((sa(j), sa(j), 0, 0.5))
            arcs.append((sa(j), sb(j), 1, 0.5))
            arcs.append((sb(j), sb(j), 1, 0.5))
            arcs.append((sb(j), a(j + 1), pa(j + 1), 0.5))
    arr = np.asarray(arcs, dtype=np.float64)
    init = np.zeros(S, dtype=np.float32); init[0] = 1.0
    fin = np.zeros(S, dtype=np.float32); fin[b(n - 1)] = 1.0
    return {
        "num_states": S,
        "num_pdfs": int(num_pdfs),
        "src": arr[:, 0].astype(np.int32),
        "dst": arr[:, 1].astype(np.int32),
        "pdf": arr[:, 2].astype(np.int32),
        "logw": np.log(arr[:, 3]).astype(np.float32),
        "init_prob": init,
        "final_prob": fin,
    }


def hmm_den_graph(rng, num_phones=42, successors=24, dirichlet=0.5):
    """Denominator-like graph expanded from two-state phone HMMs whose states emit
    (the topology of Section 4.2 without its skip): one pair of states (a, b) per
    allowed phone pair (previous phone h, phone k); arcs a->a, a->b, b->b, and from
    b of (h, k) to a of (k, k') for every allowed successor k' of k. Every arc
    carries the pdf-id of the state it enters (a-state of phone k: 2k, b-state:
    2k + 1), so the pdf-id is a function of the to-state. Each phone has
    `successors` allowed successors drawn without replacement; the out-weights of
    a state are one Dirichlet(dirichlet) draw floored at 1e-30. Uniform initial
    probability, every state final."""
    K, m = int(num_phones), int(successors)
    succ = [np.sort(rng.choice(K, size=m, replace=False)) for _ in range(K)]
    pair_id = {}
    for h in range(K):
        for k in succ[h]:
            pair_id[(h, int(k))] = len(pair_id)
    S = 2 * len(pair_id)
    src, dst, pdf = [], [], []
    for (h, k), i in pair_id.items():
        a, b = 2 * i, 2 * i + 1
        src += [a, a, b]
        dst += [a, b, b]
        pdf += [2 * k, 2 * k + 1, 2 * k + 1]
        for k2 in succ[k]:
            src.append(b)
            dst.append(2 * pair_id[(k, int(k2))])
            pdf.append(2 * int(k2))
    src = np.asarray(src, dtype=np.int32)
    dst = np.asarray(dst, dtype=np.int32)
    w = np.empty(len(src), dtype=np.float64)
    order = np.argsort(src, kind="stable")
    counts = np.bincount(src, minlength=S)
    at = 0
    for s_ in range(S):
        n = int(counts[s_])
        w[order[at:at + n]] = np.maximum(rng.dirichlet(np.full(n, float(dirichlet))), 1e-30)
        at += n
    return {
        "num_states": S,
        "num_pdfs": 2 * K,
        "src": src,
        "dst": dst,
        "pdf": np.asarray(pdf, dtype=np.int32),
        "logw": np.log(w).astype(np.float32),
        "init_prob": np.full(S, 1.0 / S, dtype=np.float32),
        "final_prob": np.ones(S, dtype=np.float32),
    }


def random_logits(rng, lengths, num_pdfs, sigma, pad_value=None):
    """float32 N(0, sigma) logits [B, max(lengths), P]. If pad_value is given
    the rows at and after each sequence's length are overwritten with it (the
    method must never read them)."""
    lengths = np.asarray(lengths)
    B, T = len(lengths), int(lengths.max())
    x = rng.standard_normal(size=(B, T, num_pdfs), dtype=np.float32)
    x *= np.float32(sigma)
    if pad_value is not None:
        for b in range(B):
            x[b, lengths[b]:, :] = pad_value
    return x


def spike_frames(rng, logits, lengths, fraction=0.01, magnitude=30.0):
    """In round(fraction * sum(lengths)) distinct valid frames, set one uniformly
    chosen pdf's logit to +magnitude (even draws) or -magnitude (odd draws)."""
    lengths = np.asarray(lengths)
    offs = np.concatenate([[0], np.cumsum(lengths)])
    total = int(offs[-1])
    n = int(round(fraction * total))
    flat = rng.choice(total, size=n, replace=False)
    pdfs = rng.integers(0, logits.shape[2], size=n)
    for k in range(n):
        b = int(np.searchsorted(offs, flat[k], side="right") - 1)
        t = int(flat[k] - offs[b])
        logits[b, t, pdfs[k]] = magnitude if k % 2 == 0 else -magnitude
    return n


def make_workload(config, seed=None, scale=None, pad_value=None):
    """Build config 1..5 (the named workloads) or 6, 7 (see below).

    `scale` (dict) overrides sizes for reduced parity cases that keep the
    structure of the named config: keys S, k, P, B, Tlo, Thi, nlo, nhi.
    """
    config = int(config)
    sc = dict(scale or {})
    rng = np.random.default_rng(BASE_SEED + config if seed is None else seed)
    name = CONFIG_NAMES[config] + ("" if not sc else "_scaled")
    leak = 1e-5
    num = None
    if config == 1:
        S, k, P, dirich = sc.get("S", 20), sc.get("k", 2), sc.get("P", 10), 1.0
        den = random_den_graph(rng, S, k, P, dirich)
        lengths = np.asarray(sc.get("lengths", [30, 25]), dtype=np.int32)
        num = [chain_num_graph(rng, sc.get("K", 8), P) for _ in lengths]
        logits = random_logits(rng, lengths, P, 1.0, pad_value)
    elif config == 2:
        S, k, P = sc.get("S", 2000), sc.get("k", 9), sc.get("P", 84)
        den = random_den_graph(rng, S, k, P, 0.5)
        B = sc.get("B", 64)
        lengths = rng.integers(sc.get("Tlo", 100), sc.get("Thi", 500) + 1, size=B)
        lengths = np.sort(lengths)[::-1].astype(np.int32)
        logits = random_logits(rng, lengths, P, 2.0, pad_value)
    elif config == 3:
        S, k, P = sc.get("S", 10000), sc.get("k", 9), sc.get("P", 3000)
        den = random_den_graph(rng, S, k, P, 0.5, pdf_dist="zipf")
        B = sc.get("B", 128)
        lengths = rng.integers(sc.get("Tlo", 150), sc.get("Thi", 500) + 1,
                               size=B).astype(np.int32)
        logits = random_logits(rng, lengths, P, 2.0, pad_value)
    elif config == 4:
        S, k, P = sc.get("S", 5000), sc.get("k", 9), sc.get("P", 84)
        den = random_den_graph(rng, S, k, P, 0.5)
        B = sc.get("B", 32)
        lengths = rng.integers(sc.get("Tlo", 200), sc.get("Thi", 1600) + 1,
                               size=B).astype(np.int32)
        logits = random_logits(rng, lengths, P, 3.0, pad_value)
        spike_frames(rng, logits, lengths, 0.01, 30.0)
    elif config == 5:
        S, k, P = sc.get("S", 2000), sc.get("k", 9), 84
        # the denominator graph is the config-2 graph (same seed, same draws)
        den = random_den_graph(np.random.default_rng(BASE_SEED + 2), S, k, P, 0.5)
        B = sc.get("B", 128)
        nph = rng.integers(sc.get("nlo", 20), sc.get("nhi", 120) + 1, size=B)
        lengths = np.asarray([rng.integers(3 * n, 5 * n + 1) for n in nph],
                             dtype=np.int32)
        num = []
        for n in nph:
            phones = rng.integers(1, 42, size=int(n))
            num.append(phone_string_num_graph(phones, P, 0.2))
        logits = random_logits(rng, lengths, P, 2.0, pad_value)
    elif config == 6:
        # Beyond the five named workloads: the shape of config 2 (about 2,000 states,
        # 84 pdfs, B = 64, T in [100, 500] sorted, N(0, 2) logits) on a graph expanded
        # from phone HMMs, where every arc carries the pdf-id of the state it enters.
        den = hmm_den_graph(rng, sc.get("phones", 42), sc.get("succ", 24), 0.5)
        P = den["num_pdfs"]
        B = sc.get("B", 64)
        lengths = rng.integers(sc.get("Tlo", 100), sc.get("Thi", 500) + 1, size=B)
        lengths = np.sort(lengths)[::-1].astype(np.int32)
        logits = random_logits(rng, lengths, P, 2.0, pad_value)
    elif config == 7:
        # Beyond the five named workloads: the sizes Section 4.4 gives for the paper's own
        # run - a denominator graph of 7,398 states, 128 sequences per batch (946,944
        # (sequence, state) pairs per time step), 84 pdfs - with what it does not give
        # filled in as in config 2: a self-loop plus 9 random out-arcs per state,
        # Dirichlet(0.5) weights, pdf-ids uniform per arc, T uniform in [100, 500].
        S, k, P = sc.get("S", 7398), sc.get("k", 9), sc.get("P", 84)
        den = random_den_graph(rng, S, k, P, 0.5)
        B = sc.get("B", 128)
        lengths = rng.integers(sc.get("Tlo", 100), sc.get("Thi", 500) + 1,
                               size=B).astype(np.int32)
        logits = random_logits(rng, lengths, P, 2.0, pad_value)
    else:
        raise ValueError("config must be 1..7")
    return {
        "name": name,
        "config": config,
        "leak": leak,
        "den": den,
        "num": num,
        "logits": logits,
        "lengths": lengths.astype(np.int32),
    }
