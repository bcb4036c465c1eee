"""Independent small-scale formulations used to pin the oracle.

None of this is the oracle's code: the brute force walks explicit paths (with
the leak as an explicit path choice), the dense twin multiplies explicit S x S
matrices in the probability domain.
"""
import itertools

import numpy as np


def small_graph(S, P, arcs, init, final):
    """arcs: list of (src, dst, pdf, weight)."""
    a = np.asarray(arcs, dtype=np.float64).reshape(-1, 4)
    return {
        "num_states": S,
        "num_pdfs": P,
        "src": a[:, 0].astype(np.int32),
        "dst": a[:, 1].astype(np.int32),
        "pdf": a[:, 2].astype(np.int32),
        "logw": np.log(a[:, 3]).astype(np.float32),
        "init_prob": np.asarray(init, dtype=np.float32),
        "final_prob": np.asarray(final, dtype=np.float32),
    }


def brute_force(graph, x, leak):
    """Sum over explicit paths. A path picks a start state, then at t = 0 and
    after each of the T arcs either stays put (weight 1) or restarts into any
    state j with weight leak * init_prob[j]. Returns (Z, gamma[T, P])."""
    S, P = graph["num_states"], graph["num_pdfs"]
    src, dst, pdf = graph["src"], graph["dst"], graph["pdf"]
    w = np.exp(graph["logw"].astype(np.float64))
    pi = graph["init_prob"].astype(np.float64)
    fin = graph["final_prob"].astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    out_arcs = [[a for a in range(len(src)) if src[a] == s] for s in range(S)]
    Z = 0.0
    gamma = np.zeros((T, P))

    def leak_moves(s):
        yield s, 1.0
        for j in range(S):
            if leak > 0.0 and pi[j] > 0.0:
                yield j, leak * pi[j]

    def walk(t, s, weight, used):
        nonlocal Z
        if t == T:
            wt = weight * fin[s]
            if wt != 0.0:
                Z += wt
                for tt, d in enumerate(used):
                    gamma[tt, d] += wt
            return
        for a in out_arcs[s]:
            wa = weight * w[a] * np.exp(x[t, pdf[a]])
            for j, wl in leak_moves(dst[a]):
                walk(t + 1, j, wa * wl, used + [pdf[a]])

    for s0 in range(S):
        if pi[s0] == 0.0:
            continue
        for j, wl in leak_moves(s0):
            walk(0, j, pi[s0] * wl, [])
    if Z > 0:
        gamma /= Z
    return Z, gamma


def dense_twin(graph, x, leak):
    """Probability-domain fp64 product f^T L M_T L ... M_1 L pi with explicit
    dense matrices; the (S, S, D) dense transition tensor of Section 3.3.
    Returns (Z, gamma[T, P], Z from the backward recursion)."""
    S, P = graph["num_states"], graph["num_pdfs"]
    W = np.zeros((S, S, P))  # W[to, from, pdf]
    np.add.at(W, (graph["dst"], graph["src"], graph["pdf"]),
              np.exp(graph["logw"].astype(np.float64)))
    pi = graph["init_prob"].astype(np.float64)
    fin = graph["final_prob"].astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    Lk = np.eye(S) + leak * np.outer(pi, np.ones(S))
    alphas = [Lk @ pi]
    for t in range(T):
        M = W @ np.exp(x[t])
        alphas.append(Lk @ (M @ alphas[-1]))
    Z = float(fin @ alphas[T])
    beta = Lk.T @ fin
    gamma = np.zeros((T, P))
    for t in range(T, 0, -1):
        e = np.exp(x[t - 1])
        gamma[t - 1] = np.einsum("j,jid,i->d", beta, W, alphas[t - 1]) * e
        beta = Lk.T @ ((W @ e).T @ beta)
    Zb = float(pi @ beta)
    if Z > 0:
        gamma /= Z
    return Z, gamma, Zb


def random_small_graph(rng, S, P, n_arcs, one_hot_init=False, sparse_final=False):
    arcs = []
    for _ in range(n_arcs):
        arcs.append((rng.integers(S), rng.integers(S), rng.integers(P),
                     rng.uniform(0.1, 1.5)))
    if one_hot_init:
        init = np.zeros(S); init[rng.integers(S)] = 1.0
    else:
        init = rng.uniform(0.1, 1.0, S)
    fin = rng.uniform(0.1, 1.0, S)
    if sparse_final:
        fin[rng.integers(S)] = 0.0
    return small_graph(S, P, arcs, init, fin)
