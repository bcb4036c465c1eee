// Host-side packing of an HMM graph into sliced-ELL orderings (see pack.h).
#include "pack.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <queue>

namespace lfmmi {
namespace {

// Where each row goes: rows sorted by length (descending, stable), cut into
// slices of 64, slices dealt to waves longest-first onto the least loaded wave,
// then renumbered so that a wave's slices are consecutive.
struct Arrangement {
    std::vector<int32_t> pos;  // row -> slice * 64 + lane
    std::vector<int32_t> slice_width;
    std::vector<int32_t> wave_first;
    std::vector<int32_t> slice_hub;  // 1: a hub slice (all 64 lanes work for the row of lane 0)
    int32_t num_slices = 0, num_waves = 0, max_wave_slots = 0;
};

// hub[r] != 0: row r gets a slice of its own and its len[r] arcs are spread over
// the 64 lanes (a row with far more arcs than the others would otherwise make
// its slice, and so its wave, that many slots long).
Arrangement arrange(const std::vector<int32_t>& len, int waves, int extra_slots,
                    const std::vector<uint8_t>* hub = nullptr)
{
    Arrangement ar;
    const int32_t R = (int32_t)len.size();
    std::vector<int32_t> idx, hubs;
    for (int32_t r = 0; r < R; ++r) (hub && (*hub)[r] ? hubs : idx).push_back(r);
    const int32_t plain = (int32_t)idx.size();
    const int32_t plain_slices = (plain + kLanes - 1) / kLanes;
    ar.num_slices = plain_slices + (int32_t)hubs.size();
    ar.num_waves = std::max(1, std::min(waves, ar.num_slices));
    std::stable_sort(idx.begin(), idx.end(),
                     [&](int32_t a, int32_t b) { return len[a] > len[b]; });
    std::vector<int32_t> sorted_width(ar.num_slices);
    for (int32_t s = 0; s < plain_slices; ++s)
        sorted_width[s] = std::max(len[idx[(size_t)s * kLanes]] + extra_slots, 1);
    for (size_t h = 0; h < hubs.size(); ++h)
        sorted_width[plain_slices + h] = (len[hubs[h]] + kLanes - 1) / kLanes + extra_slots;
    // Widths are even, with one more padding slot where needed: the kernels load
    // the records of two slots at a time (16 bytes per lane stream at twice the rate
    // of 8), and the register-resident recursion looks for the end of a slice at
    // every other slot only.
    for (int32_t& wd : sorted_width) wd += wd & 1;

    std::vector<std::vector<int32_t>> owned(ar.num_waves);
    std::vector<int64_t> load(ar.num_waves, 0);
    for (int32_t s = 0; s < ar.num_slices; ++s) {
        int best = 0;
        for (int w = 1; w < ar.num_waves; ++w) {
            if (load[w] < load[best] ||
                (load[w] == load[best] && owned[w].size() < owned[best].size()))
                best = w;
        }
        owned[best].push_back(s);
        load[best] += sorted_width[s];
    }
    // refine: move or swap slices out of the fullest wave while that lowers its load
    for (int round = 0; round < 256; ++round) {
        int top = 0;
        for (int w = 1; w < ar.num_waves; ++w)
            if (load[w] > load[top]) top = w;
        bool improved = false;
        for (size_t a = 0; a < owned[top].size() && !improved; ++a) {
            const int64_t wa = sorted_width[owned[top][a]];
            for (int w = 0; w < ar.num_waves && !improved; ++w) {
                if (w == top) continue;
                if (load[w] + wa < load[top]) {  // move
                    owned[w].push_back(owned[top][a]);
                    owned[top].erase(owned[top].begin() + a);
                    load[w] += wa;
                    load[top] -= wa;
                    improved = true;
                    break;
                }
                for (size_t c = 0; c < owned[w].size(); ++c) {  // swap
                    const int64_t wc = sorted_width[owned[w][c]];
                    if (wc < wa && load[w] - wc + wa < load[top]) {
                        std::swap(owned[top][a], owned[w][c]);
                        load[top] += wc - wa;
                        load[w] += wa - wc;
                        improved = true;
                        break;
                    }
                }
            }
        }
        if (!improved) break;
    }
    for (int w = 0; w < ar.num_waves; ++w) std::sort(owned[w].begin(), owned[w].end());
    ar.pos.assign(R, 0);
    ar.slice_width.clear();
    ar.slice_hub.clear();
    ar.wave_first.assign(ar.num_waves + 1, 0);
    int32_t next = 0;
    for (int w = 0; w < ar.num_waves; ++w) {
        ar.wave_first[w] = next;
        for (int32_t s : owned[w]) {
            if (s >= plain_slices) {
                ar.pos[hubs[s - plain_slices]] = next * kLanes;  // lane 0 owns the row
            } else {
                for (int l = 0; l < kLanes; ++l) {
                    size_t i = (size_t)s * kLanes + l;
                    if (i < (size_t)plain) ar.pos[idx[i]] = next * kLanes + l;
                }
            }
            ar.slice_width.push_back(sorted_width[s]);
            ar.slice_hub.push_back(s >= plain_slices ? 1 : 0);
            ++next;
        }
        ar.max_wave_slots = std::max<int32_t>(ar.max_wave_slots, (int32_t)load[w]);
    }
    ar.wave_first[ar.num_waves] = next;
    return ar;
}

void start_ordering(const Arrangement& ar, int32_t num_rows, Ordering* o)
{
    o->num_rows = num_rows;
    o->num_slices = ar.num_slices;
    o->num_waves = ar.num_waves;
    o->max_wave_slots = ar.max_wave_slots;
    o->wave_first = ar.wave_first;
    o->slice_hub = ar.slice_hub;
    o->slice_off.assign(ar.num_slices + 1, 0);
    for (int32_t s = 0; s < ar.num_slices; ++s)
        o->slice_off[s + 1] = o->slice_off[s] + ar.slice_width[s];
    o->total_slots = o->slice_off[ar.num_slices];
    o->key.assign((size_t)o->total_slots * kLanes, 0u);
    o->w.assign((size_t)o->total_slots * kLanes, 0.0f);
    o->row_id.assign((size_t)ar.num_slices * kLanes, -1);
}

inline void put(Ordering* o, int32_t position, int32_t nth, uint32_t x, uint32_t y, float w)
{
    const int32_t slice = position / kLanes, lane = position % kLanes;
    const size_t at = (size_t)(o->slice_off[slice] + nth) * kLanes + lane;
    o->key[at] = (x * 4u) | ((y * 4u) << 16);
    o->w[at] = w;
}


// wave_mask[w]: bit i set when slot i of wave w closes a slice; wave_hub[w]: the
// same bit when that slice is a hub slice.
void fill_wave_mask(Ordering* o)
{
    o->wave_mask.assign(o->num_waves, 0);
    o->wave_hub.assign(o->num_waves, 0);
    for (int32_t wv = 0; wv < o->num_waves; ++wv) {
        const int32_t first = o->slice_off[o->wave_first[wv]];
        const int32_t count = o->slice_off[o->wave_first[wv + 1]] - first;
        if (count > 64) continue;
        for (int32_t sl = o->wave_first[wv]; sl < o->wave_first[wv + 1]; ++sl) {
            const uint64_t bit = (uint64_t)1 << (o->slice_off[sl + 1] - 1 - first);
            o->wave_mask[wv] |= bit;
            if (o->slice_hub[sl]) o->wave_hub[wv] |= bit;
        }
    }
}

// ---- LDS bank conflicts -------------------------------------------------------
// A wave's gather is served half-wave by half-wave (32 lanes); within a half,
// lanes that hit the same one of the 32 four-byte banks at different addresses
// are served one after the other. Two things are free at pack time: which lane
// of its half-slice a state owns (its bank, as a gathered value), and the order
// of a row's arcs over the slots.

constexpr int kBanks = 32;
constexpr int kHalf = 32;

struct Lcg {
    uint64_t s;
    explicit Lcg(uint64_t seed) : s(seed * 2862933555777941757ULL + 3037000493ULL) {}
    uint32_t next() { s = s * 6364136223846793005ULL + 1442695040888963407ULL; return (uint32_t)(s >> 33); }
    uint32_t below(uint32_t n) { return (uint32_t)(((uint64_t)next() * n) >> 31) % n; }
};

// Moves states between rows so that, for each half-slice of rows, the states its
// arcs gather are spread evenly over the banks. Two states may trade places
// when each fits the other's slice (its arcs within that slice's arc slots), so
// both the bank a state is gathered from and the company its row keeps are
// free; hill climbing on the sum of squared (half-slice, bank) loads.
// row_state[a] / x_state[a]: the state that owns the row of arc a / the state
// whose value arc a gathers. pos: state -> slice * 64 + lane (updated).
// deg[s]: arcs of the row of state s; room[slice]: arc slots of the slice;
// fixed[s] != 0: the state stays where it is (hub rows).
void balance_banks(const std::vector<int32_t>& row_state, const std::vector<int32_t>& x_state,
                   const std::vector<int32_t>& deg, const std::vector<int32_t>& room,
                   const std::vector<uint8_t>& fixed, std::vector<int32_t>* pos)
{
    const int64_t A = (int64_t)row_state.size();
    const int32_t S = (int32_t)pos->size();
    if (A < 256 || S < 2 * kHalf) return;
    int32_t halves = 0;
    for (int32_t s = 0; s < S; ++s) halves = std::max(halves, (*pos)[s] / kHalf + 1);
    // per state: the states its row gathers, and the states whose rows gather it
    // (arcs of fixed rows are left out: a hub's arcs are dealt over a whole slice)
    std::vector<int32_t> out_first(S + 1, 0), in_first(S + 1, 0);
    for (int64_t a = 0; a < A; ++a)
        if (!fixed[row_state[a]]) {
            ++out_first[row_state[a] + 1];
            ++in_first[x_state[a] + 1];
        }
    for (int32_t s = 0; s < S; ++s) {
        out_first[s + 1] += out_first[s];
        in_first[s + 1] += in_first[s];
    }
    std::vector<int32_t> out_of(out_first[S]), in_of(in_first[S]);
    {
        std::vector<int32_t> fo(out_first.begin(), out_first.end() - 1),
            fi(in_first.begin(), in_first.end() - 1);
        for (int64_t a = 0; a < A; ++a)
            if (!fixed[row_state[a]]) {
                out_of[fo[row_state[a]]++] = x_state[a];
                in_of[fi[x_state[a]]++] = row_state[a];
            }
    }
    std::vector<int32_t> load((size_t)halves * kBanks, 0);
    for (int32_t s = 0; s < S; ++s)
        for (int32_t i = out_first[s]; i < out_first[s + 1]; ++i)
            ++load[(size_t)((*pos)[s] / kHalf) * kBanks + (*pos)[out_of[i]] % kBanks];

    int64_t delta = 0;
    auto add = [&](int32_t half, int32_t bank, int k) {
        int32_t& x = load[(size_t)half * kBanks + bank];
        delta += (int64_t)(x + k) * (x + k) - (int64_t)x * x;
        x += k;
    };
    // every load entry that involves u or v, taken out (k = -1) or put in (+1)
    auto touch = [&](int32_t u, int32_t v, int k) {
        for (int32_t st : {u, v}) {
            const int32_t half = (*pos)[st] / kHalf;
            for (int32_t i = out_first[st]; i < out_first[st + 1]; ++i)
                add(half, (*pos)[out_of[i]] % kBanks, k);
            const int32_t bank = (*pos)[st] % kBanks;
            for (int32_t i = in_first[st]; i < in_first[st + 1]; ++i)
                if (in_of[i] != u && in_of[i] != v)  // their rows were handled above
                    add((*pos)[in_of[i]] / kHalf, bank, k);
        }
    };
    Lcg rng(0x5eed0000u + (uint64_t)A);
    const int64_t tries = std::min<int64_t>(150LL * S, 3000000);
    for (int64_t it = 0; it < tries; ++it) {
        const int32_t u = (int32_t)rng.below((uint32_t)S), v = (int32_t)rng.below((uint32_t)S);
        if (u == v || fixed[u] || fixed[v]) continue;
        const int32_t su = (*pos)[u] / kLanes, sv = (*pos)[v] / kLanes;
        if (su != sv && (deg[u] > room[sv] || deg[v] > room[su])) continue;
        delta = 0;
        touch(u, v, -1);
        std::swap((*pos)[u], (*pos)[v]);
        touch(u, v, +1);
        if (delta > 0) {  // undo
            touch(u, v, -1);
            std::swap((*pos)[u], (*pos)[v]);
            touch(u, v, +1);
        }
    }
}

// Single-gather slot order by bipartite edge colouring. Rows and banks of one
// half-slice form a bipartite multigraph (one edge per arc); a proper colouring
// with W colours puts at most one arc of every row and of every bank node into
// each slot. A bank that gathers more than W arcs is split into several nodes of
// at most W arcs, so it shows up that many times in some slots and once in the
// others. slot_of[i] receives the colour of arc i (rows[i] in 0..31, banks[i]
// in 0..31).
void colour_half_slice(const std::vector<int32_t>& rows, const std::vector<int32_t>& banks,
                       int32_t W, std::vector<int32_t>* slot_of)
{
    const int32_t n = (int32_t)rows.size();
    slot_of->assign(n, -1);
    if (n == 0 || W == 0) return;
    // bank nodes: bank b, copy k -> node id; arcs of a bank fill copy 0 first
    std::vector<int32_t> node_of(n), seen(kBanks, 0), first_node(kBanks + 1, 0);
    std::vector<int32_t> demand(kBanks, 0);
    for (int32_t i = 0; i < n; ++i) ++demand[banks[i]];
    for (int b = 0; b < kBanks; ++b)
        first_node[b + 1] = first_node[b] + std::max(1, (demand[b] + W - 1) / W);
    for (int32_t i = 0; i < n; ++i) node_of[i] = first_node[banks[i]] + seen[banks[i]]++ / W;
    const int32_t nodes = first_node[kBanks];
    std::vector<int32_t> at_row((size_t)kHalf * W, -1), at_node((size_t)nodes * W, -1);
    auto free_colour = [&](const std::vector<int32_t>& tab, int32_t who) {
        for (int32_t c = 0; c < W; ++c)
            if (tab[(size_t)who * W + c] < 0) return c;
        return (int32_t)-1;
    };
    // Arcs of the extra nodes of overloaded banks go first: with every colour
    // still free they all land in the lowest colours, so that the slots in which
    // some bank shows up twice are shared between the overloaded banks.
    std::vector<int32_t> order;
    order.reserve(n);
    for (int32_t e = 0; e < n; ++e)
        if (node_of[e] != first_node[banks[e]]) order.push_back(e);
    for (int32_t e = 0; e < n; ++e)
        if (node_of[e] == first_node[banks[e]]) order.push_back(e);
    for (int32_t e : order) {
        const int32_t u = rows[e], v = node_of[e];
        const int32_t a = free_colour(at_row, u);   // free at the row
        const int32_t b = free_colour(at_node, v);  // free at the bank node
        if (a < 0 || b < 0) continue;               // cannot happen: degrees are <= W
        if (at_node[(size_t)v * W + a] >= 0) {
            // a is taken at v: flip the a/b alternating path that starts at v
            std::vector<int32_t> path;
            int32_t cur_is_node = 1, who = v, want = a;
            while (true) {
                const int32_t f = cur_is_node ? at_node[(size_t)who * W + want]
                                              : at_row[(size_t)who * W + want];
                if (f < 0) break;
                path.push_back(f);
                who = cur_is_node ? rows[f] : node_of[f];
                cur_is_node ^= 1;
                want = want == a ? b : a;
            }
            for (int32_t f : path) {
                const int32_t c = (*slot_of)[f];
                at_row[(size_t)rows[f] * W + c] = -1;
                at_node[(size_t)node_of[f] * W + c] = -1;
            }
            for (int32_t f : path) {
                const int32_t c = (*slot_of)[f] == a ? b : a;
                (*slot_of)[f] = c;
                at_row[(size_t)rows[f] * W + c] = f;
                at_node[(size_t)node_of[f] * W + c] = f;
            }
        }
        (*slot_of)[e] = a;
        at_row[(size_t)u * W + a] = e;
        at_node[(size_t)v * W + a] = e;
    }
}

// Slot order of one half-slice with the fewest conflict cycles a single gather can
// have: max(W, largest bank load). With k = largest load - W, k slots are set
// aside in which a bank may show up twice and W - k in which it shows up once.
// Which arcs go into the k slots is a degree-constrained subgraph: a row keeps
// at most W - k arcs for the other slots, and so does a bank, while the k slots
// hold at most k arcs of a row and 2k of a bank; found as a feasible flow
// (lower bounds by the usual excess / deficit construction, augmenting paths by
// BFS: the graph has 66 nodes). Both parts are then edge-coloured exactly.
// Returns false when no k <= W works (a bank with more than 2W arcs).
bool colour_balanced(const std::vector<int32_t>& rows, const std::vector<int32_t>& banks,
                     int32_t W, std::vector<int32_t>* slot_of)
{
    const int32_t n = (int32_t)rows.size();
    std::vector<int32_t> deg_r(kHalf, 0), deg_b(kBanks, 0);
    for (int32_t i = 0; i < n; ++i) {
        ++deg_r[rows[i]];
        ++deg_b[banks[i]];
    }
    int32_t most = 0;
    for (int b = 0; b < kBanks; ++b) most = std::max(most, deg_b[b]);
    for (int r = 0; r < kHalf; ++r)
        if (deg_r[r] > W) return false;
    if (most <= W) {  // an exact colouring has no conflict at all
        colour_half_slice(rows, banks, W, slot_of);
        for (int32_t i = 0; i < n; ++i)
            if ((*slot_of)[i] < 0) return false;
        return true;
    }
    // nodes: 0 source, 1 sink, 2 + r rows, 2 + kHalf + b banks, then super source / sink
    constexpr int kSrc = 0, kSnk = 1, kRow0 = 2, kBank0 = 2 + kHalf, kSS = kBank0 + kBanks,
                  kTT = kSS + 1, kNodes = kTT + 1;
    struct Edge { int32_t to, cap, arc; };
    for (int32_t k = most - W; k <= W; ++k) {
        std::vector<Edge> edges;
        std::vector<std::vector<int32_t>> adj(kNodes);
        auto add_edge = [&](int32_t u, int32_t v, int32_t cap, int32_t arc) {
            adj[u].push_back((int32_t)edges.size());
            edges.push_back({v, cap, arc});
            adj[v].push_back((int32_t)edges.size());
            edges.push_back({u, 0, -1});
        };
        std::vector<int32_t> excess(kNodes, 0);
        bool possible = true;
        auto bounded = [&](int32_t u, int32_t v, int32_t lo, int32_t hi) {
            if (lo > hi) { possible = false; return; }
            excess[v] += lo;
            excess[u] -= lo;
            add_edge(u, v, hi - lo, -1);
        };
        for (int r = 0; r < kHalf; ++r)
            bounded(kSrc, kRow0 + r, std::max(0, deg_r[r] - (W - k)), std::min(k, deg_r[r]));
        for (int b = 0; b < kBanks; ++b)
            bounded(kBank0 + b, kSnk, std::max(0, deg_b[b] - (W - k)), std::min(2 * k, deg_b[b]));
        if (!possible) continue;
        for (int32_t i = 0; i < n; ++i) add_edge(kRow0 + rows[i], kBank0 + banks[i], 1, i);
        add_edge(kSnk, kSrc, 1 << 28, -1);
        int32_t need = 0;
        for (int v = 0; v < kNodes; ++v) {
            if (excess[v] > 0) { add_edge(kSS, v, excess[v], -1); need += excess[v]; }
            if (excess[v] < 0) add_edge(v, kTT, -excess[v], -1);
        }
        int32_t flow = 0;
        while (true) {  // shortest augmenting paths
            std::vector<int32_t> via(kNodes, -1), queue{kSS};
            via[kSS] = -2;
            for (size_t q = 0; q < queue.size() && via[kTT] == -1; ++q)
                for (int32_t e : adj[queue[q]])
                    if (edges[e].cap > 0 && via[edges[e].to] == -1) {
                        via[edges[e].to] = e;
                        queue.push_back(edges[e].to);
                    }
            if (via[kTT] == -1) break;
            int32_t push = 1 << 28;
            for (int32_t v = kTT; v != kSS; v = edges[via[v] ^ 1].to) push = std::min(push, edges[via[v]].cap);
            for (int32_t v = kTT; v != kSS; v = edges[via[v] ^ 1].to) {
                edges[via[v]].cap -= push;
                edges[via[v] ^ 1].cap += push;
            }
            flow += push;
        }
        if (flow != need) continue;
        // arcs that carry flow go into the k shared slots
        std::vector<int32_t> part(n, 0);
        for (const Edge& e : edges)
            if (e.arc >= 0 && e.cap == 0) part[e.arc] = 1;
        std::vector<int32_t> sub_rows[2], sub_banks[2], sub_arc[2], col;
        for (int32_t i = 0; i < n; ++i) {
            sub_rows[part[i]].push_back(rows[i]);
            sub_banks[part[i]].push_back(banks[i]);
            sub_arc[part[i]].push_back(i);
        }
        slot_of->assign(n, -1);
        bool ok = true;
        for (int which = 0; which < 2 && ok; ++which) {
            const int32_t width = which == 0 ? W - k : k, first = which == 0 ? 0 : W - k;
            if (sub_arc[which].empty()) continue;
            if (width <= 0) { ok = false; break; }
            colour_half_slice(sub_rows[which], sub_banks[which], width, &col);
            for (size_t i = 0; i < sub_arc[which].size(); ++i) {
                if (col[i] < 0) ok = false;
                (*slot_of)[sub_arc[which][i]] = first + col[i];
            }
        }
        if (ok) return true;
    }
    return false;
}

// Chooses the slot (0 .. width - 1 inside its slice) of every arc. pos_row[a]:
// position of the arc's row; ax[a], ay[a]: the words its two gathers read (bank =
// word % 32), -1 for a gather that cannot conflict. width[slice]: arc slots of
// the slice. Lanes of a half-wave that read the same word do not conflict (the
// word is broadcast), so what is balanced over the banks of a slot is the number
// of distinct words, not of arcs: with skewed pdf-ids, or a state many arcs
// leave, most reads of a bank are of one word.
void order_slots(const std::vector<int32_t>& pos_row, const std::vector<int32_t>& ax,
                 const std::vector<int32_t>& ay, int32_t num_slices,
                 const std::vector<int32_t>& width, std::vector<int32_t>* nth)
{
    const int64_t A = (int64_t)pos_row.size();
    nth->assign(A, 0);
    const int32_t halves = num_slices * 2;
    std::vector<std::vector<int32_t>> arcs_of(halves);
    for (int64_t a = 0; a < A; ++a) arcs_of[pos_row[a] / kHalf].push_back((int32_t)a);
    Lcg rng(0xb0a7u + (uint64_t)A);
    std::vector<int32_t> slot_of;      // per arc of the half-slice
    std::vector<int32_t> table;        // [row][slot] -> local arc index or -1
    std::vector<int32_t> lx, ly;       // [slot][bank]: distinct words read there
    std::vector<int32_t> ux, uy;       // the half-slice's distinct words, sorted
    std::vector<int32_t> idx, idy;     // per arc: index of its word in ux / uy, or -1
    std::vector<uint16_t> cx, cy;      // [slot][word index]: arcs that read it
    for (int32_t h = 0; h < halves; ++h) {
        const std::vector<int32_t>& arcs = arcs_of[h];
        const int32_t W = width[h / 2];
        const int32_t n = (int32_t)arcs.size();
        if (n == 0 || W == 0) continue;
        if (ay[arcs[0]] < 0 && ax[arcs[0]] >= 0) {
            // one gather only: an edge colouring is (nearly) conflict-free by construction
            std::vector<int32_t> rws(n), bks(n), col;
            for (int32_t i = 0; i < n; ++i) {
                rws[i] = pos_row[arcs[i]] % kHalf;
                bks[i] = ax[arcs[i]] % kBanks;
            }
            bool ok = colour_balanced(rws, bks, W, &col);
            if (!ok) {
                colour_half_slice(rws, bks, W, &col);
                ok = true;
            }
            for (int32_t i = 0; i < n; ++i) ok = ok && col[i] >= 0;
            if (ok) {
                for (int32_t i = 0; i < n; ++i) (*nth)[arcs[i]] = col[i];
                continue;
            }
        }
        table.assign((size_t)kHalf * W, -1);
        lx.assign((size_t)W * kBanks, 0);
        ly.assign((size_t)W * kBanks, 0);
        slot_of.assign(n, -1);
        auto index_words = [&](const std::vector<int32_t>& word, std::vector<int32_t>* uniq,
                               std::vector<int32_t>* id) {
            uniq->clear();
            for (int32_t i = 0; i < n; ++i)
                if (word[arcs[i]] >= 0) uniq->push_back(word[arcs[i]]);
            std::sort(uniq->begin(), uniq->end());
            uniq->erase(std::unique(uniq->begin(), uniq->end()), uniq->end());
            id->assign(n, -1);
            for (int32_t i = 0; i < n; ++i)
                if (word[arcs[i]] >= 0)
                    (*id)[i] = (int32_t)(std::lower_bound(uniq->begin(), uniq->end(), word[arcs[i]]) -
                                         uniq->begin());
        };
        index_words(ax, &ux, &idx);
        index_words(ay, &uy, &idy);
        const size_t mx = std::max<size_t>(ux.size(), 1), my = std::max<size_t>(uy.size(), 1);
        cx.assign((size_t)W * mx, 0);
        cy.assign((size_t)W * my, 0);
        std::vector<std::vector<int32_t>> row_arcs(kHalf);
        for (int32_t i = 0; i < n; ++i) row_arcs[pos_row[arcs[i]] % kHalf].push_back(i);
        // what arc i would add to slot j: the load of its banks, unless its word is
        // read there already
        auto cost_at = [&](int32_t j, int32_t i) {
            int32_t c = 0;
            if (idx[i] >= 0 && cx[(size_t)j * mx + idx[i]] == 0)
                c += lx[(size_t)j * kBanks + ux[idx[i]] % kBanks];
            if (idy[i] >= 0 && cy[(size_t)j * my + idy[i]] == 0)
                c += ly[(size_t)j * kBanks + uy[idy[i]] % kBanks];
            return c;
        };
        auto place = [&](int32_t r, int32_t j, int32_t i, int sign) {
            if (idx[i] >= 0) {
                uint16_t& c = cx[(size_t)j * mx + idx[i]];
                int32_t& l = lx[(size_t)j * kBanks + ux[idx[i]] % kBanks];
                if (sign > 0) { if (c++ == 0) ++l; } else { if (--c == 0) --l; }
            }
            if (idy[i] >= 0) {
                uint16_t& c = cy[(size_t)j * my + idy[i]];
                int32_t& l = ly[(size_t)j * kBanks + uy[idy[i]] % kBanks];
                if (sign > 0) { if (c++ == 0) ++l; } else { if (--c == 0) --l; }
            }
            table[(size_t)r * W + j] = sign > 0 ? i : -1;
            slot_of[i] = sign > 0 ? j : -1;
        };
        // greedy: slot by slot, rows with the fewest arcs left choose first
        std::vector<int32_t> order(kHalf);
        std::vector<std::vector<int32_t>> left = row_arcs;
        for (int32_t j = 0; j < W; ++j) {
            std::iota(order.begin(), order.end(), 0);
            std::stable_sort(order.begin(), order.end(), [&](int32_t p, int32_t q) {
                return left[p].size() < left[q].size();
            });
            for (int32_t r : order) {
                std::vector<int32_t>& cand = left[r];
                if (cand.empty()) continue;
                size_t best = 0;
                int32_t best_cost = cost_at(j, cand[0]);
                for (size_t c = 1; c < cand.size(); ++c) {
                    const int32_t cc = cost_at(j, cand[c]);
                    if (cc < best_cost) { best_cost = cc; best = c; }
                }
                place(r, j, cand[best], 1);
                cand.erase(cand.begin() + best);
            }
        }
        // hill climbing on the modelled cycles of the two slots of a move (squared bank
        // loads break ties: on their own they spread conflicts over many slots, each of
        // which then costs a cycle, where the cycles want them in few): move an arc of a
        // row to another slot of that row (swapping with what is there)
        auto squares = [&](int32_t i, int32_t other, int32_t j1, int32_t j2) {
            int32_t cells[8];
            int nc = 0;
            auto add = [&](int32_t cell) {
                for (int q = 0; q < nc; ++q)
                    if (cells[q] == cell) return;
                cells[nc++] = cell;
            };
            int64_t sum = 0;
            for (int which = 0; which < 2; ++which) {
                nc = 0;
                const std::vector<int32_t>& id = which == 0 ? idx : idy;
                const std::vector<int32_t>& uq = which == 0 ? ux : uy;
                const std::vector<int32_t>& ld = which == 0 ? lx : ly;
                for (int32_t arc : {i, other}) {
                    if (arc < 0 || id[arc] < 0) continue;
                    const int32_t bank = uq[id[arc]] % kBanks;
                    add(j1 * kBanks + bank);
                    add(j2 * kBanks + bank);
                }
                for (int q = 0; q < nc; ++q) sum += (int64_t)ld[cells[q]] * ld[cells[q]];
            }
            return sum;
        };
        // what the two slots of a move cost: per gather the most loaded bank (the cycles of
        // the half-wave's read); squared loads break ties
        auto slots_cost = [&](int32_t i, int32_t other, int32_t j1, int32_t j2) {
            int64_t c = 0;
            for (const int32_t j : {j1, j2}) {
                int32_t mx_ = 0, my_ = 0;
                for (int k = 0; k < kBanks; ++k) {
                    mx_ = std::max(mx_, lx[(size_t)j * kBanks + k]);
                    my_ = std::max(my_, ly[(size_t)j * kBanks + k]);
                }
                c += mx_ + my_;
            }
            return c * 1000000 + squares(i, other, j1, j2);
        };
        const int64_t tries = 80LL * n;
        for (int64_t it = 0; it < tries; ++it) {
            const int32_t i = (int32_t)rng.below((uint32_t)n);
            const int32_t r = pos_row[arcs[i]] % kHalf;
            const int32_t j1 = slot_of[i];
            const int32_t j2 = (int32_t)rng.below((uint32_t)W);
            if (j1 == j2) continue;
            const int32_t other = table[(size_t)r * W + j2];
            const int64_t before = slots_cost(i, other, j1, j2);
            place(r, j1, i, -1);
            if (other >= 0) place(r, j2, other, -1);
            place(r, j2, i, 1);
            if (other >= 0) place(r, j1, other, 1);
            if (slots_cost(i, other, j1, j2) > before) {  // worse: back
                place(r, j2, i, -1);
                if (other >= 0) place(r, j1, other, -1);
                place(r, j1, i, 1);
                if (other >= 0) place(r, j2, other, 1);
            }
        }
        for (int32_t i = 0; i < n; ++i) (*nth)[arcs[i]] = slot_of[i];
    }
}

// (graphs with fewer arcs keep the ordered slots: the per-utterance graphs of a batch
// are packed at every call of the trainer, and have little to gain)
constexpr int64_t kDealMinArcs = 4096;

// OCC ordering: deals every arc to a row of its pdf and a slot of that row.
// pdf_of[r], len[r]: pdf and arc count of row r; ar: where the rows sit; pos_f /
// pos_b: state -> position in the FWD / BWD numbering (the words the two gathers
// of an arc read). For every half-slice, slot by slot: rows that must take an
// arc in this slot (as many arcs left as slots) choose first, then the others;
// a row takes an arc of its pdf whose two banks are still free in this slot, an
// optional row rather none than one that conflicts; a forced row takes the arc
// with the fewest conflicts, and then tries to have the rows it collides with
// take other arcs (one level of re-choosing). Deterministic.
void deal_occ_arcs(const ArcList& g, const std::vector<int32_t>& pdf_of,
                   const std::vector<int32_t>& len, const Arrangement& ar,
                   const std::vector<int32_t>& pos_f, const std::vector<int32_t>& pos_b,
                   std::vector<int32_t>* prow, std::vector<int32_t>* nth)
{
    const int64_t A = g.num_arcs;
    int32_t num_pdfs = 0;
    for (int32_t d : pdf_of) num_pdfs = std::max(num_pdfs, d + 1);
    for (int64_t a = 0; a < A; ++a) num_pdfs = std::max(num_pdfs, g.pdf[a] + 1);
    std::vector<std::vector<int32_t>> pool(num_pdfs);  // arcs of a pdf not dealt yet
    for (int64_t a = 0; a < A; ++a) pool[g.pdf[a]].push_back((int32_t)a);
    std::vector<uint8_t> taken(A, 0);
    auto bank_f = [&](int32_t a) { return pos_f[g.src[a]] % kBanks; };
    auto bank_b = [&](int32_t a) { return pos_b[g.dst[a]] % kBanks; };
    const int32_t halves = ar.num_slices * 2;
    std::vector<std::vector<int32_t>> rows_of(halves);
    for (int32_t r = 0; r < (int32_t)len.size(); ++r) rows_of[ar.pos[r] / kHalf].push_back(r);
    std::vector<int32_t> need, order, chosen;
    for (int32_t h = 0; h < halves; ++h) {
        const std::vector<int32_t>& rows = rows_of[h];
        if (rows.empty()) continue;
        const int32_t W = ar.slice_width[h / 2];
        need.assign(rows.size(), 0);
        for (size_t i = 0; i < rows.size(); ++i) need[i] = len[rows[i]];
        // the pools of this half-slice's pdfs without the arcs dealt so far
        for (int32_t r : rows) {
            std::vector<int32_t>& q = pool[pdf_of[r]];
            q.erase(std::remove_if(q.begin(), q.end(), [&](int32_t a) { return taken[a] != 0; }),
                    q.end());
        }
        for (int32_t j = 0; j < W; ++j) {
            int32_t own_f[kBanks], own_b[kBanks];  // the row that holds a bank in this slot
            std::fill(own_f, own_f + kBanks, -1);
            std::fill(own_b, own_b + kBanks, -1);
            chosen.assign(rows.size(), -1);
            // a free arc of row i's pdf whose banks nobody holds (-1: none)
            auto free_arc = [&](int32_t i) {
                for (int32_t a : pool[pdf_of[rows[i]]])
                    if (!taken[a] && own_f[bank_f(a)] < 0 && own_b[bank_b(a)] < 0) return a;
                return (int32_t)-1;
            };
            auto take = [&](int32_t i, int32_t a) {
                chosen[i] = a;
                taken[a] = 1;
                if (own_f[bank_f(a)] < 0) own_f[bank_f(a)] = i;
                if (own_b[bank_b(a)] < 0) own_b[bank_b(a)] = i;
            };
            auto drop = [&](int32_t i) {
                const int32_t a = chosen[i];
                taken[a] = 0;
                if (own_f[bank_f(a)] == i) own_f[bank_f(a)] = -1;
                if (own_b[bank_b(a)] == i) own_b[bank_b(a)] = -1;
                chosen[i] = -1;
            };
            order.resize(rows.size());
            std::iota(order.begin(), order.end(), 0);
            const int32_t slots_left = W - j;
            std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
                const bool fx = need[x] >= slots_left, fy = need[y] >= slots_left;
                return fx != fy ? fx : need[x] > need[y];
            });
            for (int32_t i : order) {
                if (need[i] <= 0) continue;
                const bool forced = need[i] >= slots_left;
                int32_t a = free_arc(i);
                if (a >= 0) {
                    take(i, a);
                    continue;
                }
                if (!forced) continue;  // rather an empty slot than a conflict
                // every free arc of the pdf collides: try each with the rows it collides
                // with (at most two) re-choosing; keep the first that leaves no conflict
                bool settled = false;
                int32_t fallback = -1;
                for (int32_t cand : pool[pdf_of[rows[i]]]) {
                    if (taken[cand]) continue;
                    if (fallback < 0) fallback = cand;
                    const int32_t l1 = own_f[bank_f(cand)], l2 = own_b[bank_b(cand)];
                    int32_t blockers[2], nb = 0, old_arc[2];
                    if (l1 >= 0) blockers[nb++] = l1;
                    if (l2 >= 0 && l2 != l1) blockers[nb++] = l2;
                    for (int q = 0; q < nb; ++q) {
                        old_arc[q] = chosen[blockers[q]];
                        drop(blockers[q]);
                    }
                    bool ok = own_f[bank_f(cand)] < 0 && own_b[bank_b(cand)] < 0;
                    int32_t placed = 0;
                    if (ok) {
                        take(i, cand);
                        for (; placed < nb; ++placed) {
                            const int32_t alt = free_arc(blockers[placed]);
                            if (alt < 0) break;
                            take(blockers[placed], alt);
                        }
                        ok = placed == nb;
                    }
                    if (ok) {
                        settled = true;
                        break;
                    }
                    // back to where it was
                    for (int32_t q = 0; q < placed; ++q) drop(blockers[q]);
                    if (chosen[i] >= 0) drop(i);
                    for (int q = 0; q < nb; ++q) take(blockers[q], old_arc[q]);
                }
                if (!settled && fallback >= 0) {
                    // the arc with the fewest collisions
                    int32_t best = fallback, best_cost = 3;
                    for (int32_t cand : pool[pdf_of[rows[i]]]) {
                        if (taken[cand]) continue;
                        const int cost = (own_f[bank_f(cand)] >= 0) + (own_b[bank_b(cand)] >= 0);
                        if (cost < best_cost) { best_cost = cost; best = cand; }
                    }
                    take(i, best);
                }
            }
            for (size_t i = 0; i < rows.size(); ++i)
                if (chosen[i] >= 0) {
                    (*prow)[chosen[i]] = ar.pos[rows[i]];
                    (*nth)[chosen[i]] = j;
                    --need[i];
                }
        }
    }
}

// Padding slots (w == 0) still gather: point each at a bank its half-wave does
// not use in that slot (or, failing that, at an address another lane reads
// anyway), so that padding never adds a bank conflict. fix_y: do the same for
// the second gather. skip_last: leave the closing slot of every slice alone.
void retarget_padding(Ordering* o, bool fix_y, bool skip_last, int32_t x_rows, int32_t y_rows)
{
    for (int32_t sl = 0; sl < o->num_slices; ++sl) {
        const int32_t j1 = o->slice_off[sl + 1] - (skip_last ? 1 : 0);
        for (int32_t j = o->slice_off[sl]; j < j1; ++j)
            for (int h = 0; h < 2; ++h)
                for (int which = 0; which < (fix_y ? 2 : 1); ++which) {
                    const int32_t limit = which == 0 ? x_rows : y_rows;
                    bool used[kBanks] = {false};
                    int32_t any = -1;
                    for (int l = 0; l < kHalf; ++l) {
                        const size_t at = (size_t)j * kLanes + h * kHalf + l;
                        if (o->w[at] == 0.f) continue;
                        const uint32_t idx =
                            which == 0 ? (o->key[at] & 0xffffu) / 4 : (o->key[at] >> 16) / 4;
                        used[idx % kBanks] = true;
                        any = (int32_t)idx;
                    }
                    int next_free = 0;
                    for (int l = 0; l < kHalf; ++l) {
                        const size_t at = (size_t)j * kLanes + h * kHalf + l;
                        if (o->w[at] != 0.f) continue;
                        while (next_free < kBanks && (used[next_free] || next_free >= limit))
                            ++next_free;
                        uint32_t idx = 0;
                        if (next_free < kBanks) {
                            idx = (uint32_t)next_free;  // bank next_free, nobody else there
                            used[next_free] = true;
                        } else if (any >= 0) {
                            idx = (uint32_t)any;        // same address as a real arc: broadcast
                        }
                        if (which == 0)
                            o->key[at] = (o->key[at] & 0xffff0000u) | (idx * 4u);
                        else
                            o->key[at] = (o->key[at] & 0x0000ffffu) | ((idx * 4u) << 16);
                    }
                }
    }
}

// Modelled LDS cycles of the x gather (and the y gather when count_y) of one
// ordering: per slot and half-wave, the largest number of distinct addresses
// that fall into one bank (at least 1).
int64_t gather_cycles(const Ordering& o, bool count_y)
{
    int64_t total = 0;
    std::vector<uint32_t> seen;
    for (int32_t sl = 0; sl < o.num_slices; ++sl)
        for (int32_t j = o.slice_off[sl]; j < o.slice_off[sl + 1]; ++j)
            for (int h = 0; h < 2; ++h)
                for (int which = 0; which < (count_y ? 2 : 1); ++which) {
                    int best = 1;
                    for (int b = 0; b < kBanks; ++b) {
                        seen.clear();
                        for (int l = 0; l < kHalf; ++l) {
                            const uint32_t key = o.key[(size_t)j * kLanes + h * kHalf + l];
                            const uint32_t idx = which == 0 ? (key & 0xffffu) / 4 : (key >> 16) / 4;
                            if ((int)(idx % kBanks) != b) continue;
                            if (std::find(seen.begin(), seen.end(), idx) == seen.end())
                                seen.push_back(idx);
                        }
                        best = std::max(best, (int)seen.size());
                    }
                    total += best;
                }
    return total;
}

}  // namespace

int choose_waves(int64_t num_arcs, int32_t num_states)
{
    // about 2 arc slots per lane before a further wave pays for its share of
    // the per-frame barriers; never more waves than slices of states
    int64_t by_arcs = (num_arcs + (int64_t)kLanes * 2 - 1) / ((int64_t)kLanes * 2);
    int64_t slices = (num_states + kLanes - 1) / kLanes;
    int64_t w = std::max<int64_t>(1, std::min<int64_t>(by_arcs, slices));
    return (int)std::min<int64_t>(w, kMaxWaves);
}

bool uniform_init(const ArcList& g)
{
    for (int32_t s = 1; s < g.num_states; ++s)
        if (g.init_prob[s] != g.init_prob[0]) return false;
    return true;
}

std::string pack_graph(const ArcList& g, int32_t num_pdfs, int rec_waves, int occ_waves,
                       bool per_arc_leak, const PackTuning& tune, PackedGraph* out,
                       bool* bad_graph)
{
    *bad_graph = false;
    const int32_t S = g.num_states;
    const int64_t A = g.num_arcs;
    if (S < 1) return "num_states must be >= 1";
    if (A < 0) return "num_arcs must be >= 0";
    if (num_pdfs < 1) return "num_pdfs must be >= 1";
    if (A > 0 && (!g.src || !g.dst || !g.pdf || !g.logw)) return "null arc array";
    if (!g.init_prob || !g.final_prob) return "null init_prob / final_prob";
    if (A > (int64_t)1 << 30) return "too many arcs";
    *bad_graph = true;
    for (int64_t a = 0; a < A; ++a) {
        if (g.src[a] < 0 || g.src[a] >= S || g.dst[a] < 0 || g.dst[a] >= S)
            return "arc " + std::to_string(a) + ": state id out of range";
        if (g.pdf[a] < 0 || g.pdf[a] >= num_pdfs)
            return "arc " + std::to_string(a) + ": pdf id out of range";
        if (!std::isfinite(g.logw[a]))
            return "arc " + std::to_string(a) + ": log weight is not finite";
    }
    for (int32_t s = 0; s < S; ++s) {
        if (!(g.init_prob[s] >= 0.f) || !std::isfinite(g.init_prob[s]))
            return "init_prob[" + std::to_string(s) + "] is negative or not finite";
        if (!(g.final_prob[s] >= 0.f) || !std::isfinite(g.final_prob[s]))
            return "final_prob[" + std::to_string(s) + "] is negative or not finite";
    }
    *bad_graph = false;

    out->num_states = S;
    out->num_arcs = A;

    // ---- FWD (rows = to-states) and BWD (rows = from-states) arrangements
    std::vector<int32_t> indeg(S, 0), outdeg(S, 0);
    for (int64_t a = 0; a < A; ++a) { ++indeg[g.dst[a]]; ++outdeg[g.src[a]]; }
    // with a uniform pi the leak-dot weights are constants and need no slot
    const int closing = per_arc_leak ? 1 : 0;
    // Hub rows: at least 64 arcs and more than four times what nine rows in ten
    // have. Such a row gets a slice of its own, its arcs dealt to the 64 lanes; the
    // kernels add the lanes' sums up where the slice ends.
    auto hubs_of = [&](const std::vector<int32_t>& deg) {
        std::vector<int32_t> sorted(deg);
        std::sort(sorted.begin(), sorted.end());
        const int64_t usual = sorted[(size_t)((int64_t)(S - 1) * 9 / 10)];
        std::vector<uint8_t> hub(S, 0);
        for (int32_t s = 0; s < S; ++s)
            hub[s] = tune.hub_slices && deg[s] >= kLanes && deg[s] > 4 * usual ? 1 : 0;
        return hub;
    };
    std::vector<uint8_t> hub_f = hubs_of(indeg), hub_b = hubs_of(outdeg);
    Arrangement af = arrange(indeg, rec_waves, closing, &hub_f);
    Arrangement ab = arrange(outdeg, rec_waves, closing, &hub_b);
    // A hub slice adds 63 padding rows. Row numbers of both orderings go into 16-bit
    // key fields (index * 4): when the padded rows of either no longer fit, the
    // graph is packed without hub slices (slower, never wrong).
    if (af.num_slices * kLanes > kMaxIndex || ab.num_slices * kLanes > kMaxIndex) {
        std::fill(hub_f.begin(), hub_f.end(), 0);
        std::fill(hub_b.begin(), hub_b.end(), 0);
        af = arrange(indeg, rec_waves, closing, &hub_f);
        ab = arrange(outdeg, rec_waves, closing, &hub_b);
    }
    if (af.num_slices * kLanes > kMaxIndex || ab.num_slices * kLanes > kMaxIndex)
        return "too many states";
    std::vector<int32_t> vsrc(g.src, g.src + A), vdst(g.dst, g.dst + A);
    if (tune.balance_banks) {
        std::vector<int32_t> room_f(af.slice_width), room_b(ab.slice_width);
        for (int32_t& r : room_f) r -= closing;
        for (int32_t& r : room_b) r -= closing;
        // alpha gathers from-states in FWD numbering, beta to-states in BWD numbering
        balance_banks(vdst, vsrc, indeg, room_f, hub_f, &af.pos);
        balance_banks(vsrc, vdst, outdeg, room_b, hub_b, &ab.pos);
    }
    start_ordering(af, S, &out->ord[0]);
    start_ordering(ab, S, &out->ord[1]);
    for (int32_t s = 0; s < S; ++s) {
        out->ord[0].row_id[af.pos[s]] = s;
        out->ord[1].row_id[ab.pos[s]] = s;
    }
    std::vector<float> w(A);
    for (int64_t a = 0; a < A; ++a) w[a] = (float)std::exp((double)g.logw[a]);
    // slot of every arc inside its row, per ordering
    std::vector<int32_t> nth_f(A), nth_b(A);
    // position (slice * 64 + lane) of the row an arc is stored in: its state's row,
    // or for a hub the next of the 64 lanes of the hub's slice
    std::vector<int32_t> prow_f(A), prow_b(A);
    {
        std::vector<int32_t> wf(af.num_slices), wb_(ab.num_slices), dealt_f(S, 0), dealt_b(S, 0);
        std::vector<int32_t> bxf(A), bxb(A), byy(A);  // the words the gathers read
        for (int64_t a = 0; a < A; ++a) {
            const int32_t i = g.src[a], j = g.dst[a];
            prow_f[a] = af.pos[j] + (hub_f[j] ? dealt_f[j]++ % kLanes : 0);
            prow_b[a] = ab.pos[i] + (hub_b[i] ? dealt_b[i]++ % kLanes : 0);
            bxf[a] = af.pos[g.src[a]];
            bxb[a] = ab.pos[g.dst[a]];
            byy[a] = tune.emission_conflicts ? g.pdf[a] : -1;
        }
        for (int32_t sl = 0; sl < af.num_slices; ++sl) wf[sl] = af.slice_width[sl] - closing;
        for (int32_t sl = 0; sl < ab.num_slices; ++sl) wb_[sl] = ab.slice_width[sl] - closing;
        if (tune.order_slots) {
            order_slots(prow_f, bxf, byy, af.num_slices, wf, &nth_f);
            order_slots(prow_b, bxb, byy, ab.num_slices, wb_, &nth_b);
        } else {
            std::vector<int32_t> nf((size_t)af.num_slices * kLanes, 0),
                nb((size_t)ab.num_slices * kLanes, 0);
            for (int64_t a = 0; a < A; ++a) {
                nth_f[a] = nf[prow_f[a]]++;
                nth_b[a] = nb[prow_b[a]]++;
            }
        }
        for (int64_t a = 0; a < A; ++a) {
            const int32_t i = g.src[a], j = g.dst[a];
            put(&out->ord[0], prow_f[a], nth_f[a], (uint32_t)af.pos[i], (uint32_t)g.pdf[a], w[a]);
            put(&out->ord[1], prow_b[a], nth_b[a], (uint32_t)ab.pos[j], (uint32_t)g.pdf[a], w[a]);
        }
    }

    // ---- per-direction vectors in row numbering
    for (int d = 0; d < 2; ++d) {
        const Arrangement& ar = d == 0 ? af : ab;
        const size_t n = (size_t)ar.num_slices * kLanes;
        out->vinit[d].assign(n, 0.f);
        out->va[d].assign(n, 0.f);
        out->vb[d].assign(n, 0.f);
        out->vfin[d].assign(n, 0.f);
        for (int32_t s = 0; s < S; ++s) {
            const int32_t p = ar.pos[s];
            const float pi = g.init_prob[s], fin = g.final_prob[s];
            out->vinit[d][p] = d == 0 ? pi : fin;
            out->vfin[d][p] = d == 0 ? fin : pi;
            out->va[d][p] = d == 0 ? 1.f : pi;
            out->vb[d][p] = d == 0 ? pi : 1.f;
        }
        // closing slot of every slice: the row's leak-dot weight
        Ordering& o = out->ord[d];
        o.closing_slots = closing;
        o.a_const = d == 0 ? 1.f : g.init_prob[0];
        if (closing)
            for (int32_t sl = 0; sl < o.num_slices; ++sl)
                for (int l = 0; l < kLanes; ++l) {
                    const size_t at = (size_t)(o.slice_off[sl + 1] - 1) * kLanes + l;
                    o.key[at] = 0u;
                    o.w[at] = out->va[d][(size_t)sl * kLanes + l];
                }
        fill_wave_mask(&o);
    }
    // ---- is the pdf-id of an arc a function of the state it enters?
    {
        std::vector<int32_t> pdf_of(S, -1);
        bool by_dst = true;
        for (int64_t a = 0; a < A && by_dst; ++a) {
            int32_t& q = pdf_of[g.dst[a]];
            if (q < 0) q = g.pdf[a];
            else by_dst = q == g.pdf[a];
        }
        out->pdf_by_dst = by_dst;
        for (int d = 0; d < 2; ++d) {
            out->row_pdf[d].clear();
            if (!by_dst) continue;
            const Arrangement& ar = d == 0 ? af : ab;
            out->row_pdf[d].assign((size_t)ar.num_slices * kLanes, 0);
            for (int32_t s = 0; s < S; ++s) out->row_pdf[d][ar.pos[s]] = std::max(pdf_of[s], 0);
        }
    }
    // leak target: BWD adds the same amount to every state; FWD adds pi, which
    // is one constant when pi is uniform. Otherwise (or when another graph of
    // the same handle needs it) every arc carries the factor w * b[from]
    // (FWD: w * pi[from]; BWD: w), so that all of them run the same code.
    {
        const bool uniform = uniform_init(g);
        if (!uniform && !per_arc_leak) return "internal: per-arc leak factors are required";
        out->ord[0].has_wb = per_arc_leak ? 1 : 0;
        out->ord[0].b_const = uniform ? g.init_prob[0] : 0.f;
        out->ord[1].has_wb = per_arc_leak ? 1 : 0;
        out->ord[1].b_const = 1.f;
        if (per_arc_leak) {
            Ordering& of = out->ord[0];
            Ordering& ob = out->ord[1];
            of.wb.assign(of.w.size(), 0.f);
            ob.wb.assign(ob.w.size(), 0.f);
            for (int64_t a = 0; a < A; ++a) {
                const int32_t i = g.src[a];
                const int32_t pf = prow_f[a], pb = prow_b[a];
                of.wb[(size_t)(of.slice_off[pf / kLanes] + nth_f[a]) * kLanes + pf % kLanes] =
                    w[a] * g.init_prob[i];
                ob.wb[(size_t)(ob.slice_off[pb / kLanes] + nth_b[a]) * kLanes + pb % kLanes] = w[a];
            }
        }
    }

    // ---- OCC: arcs grouped by pdf, each pdf's list cut into pieces
    {
        std::vector<int64_t> count(num_pdfs, 0);
        for (int64_t a = 0; a < A; ++a) ++count[g.pdf[a]];
        // Every row's sum takes an LDS word per frame in flight, so rows are kept
        // few: k slices per wave, i.e. waves * 64 * k rows, handed to the pdfs one
        // at a time, always to the pdf whose pieces are longest at that moment. A
        // pdf's pieces then differ by at most one arc, and sorting rows by length
        // leaves little padding. k: the smallest whose fullest wave is within 8 %
        // of the best over all k tried (rows cost LDS: fewer of them can let a
        // second workgroup share the compute unit).
        const int waves_o = std::max(1, occ_waves);
        int64_t nonempty = 0;
        for (int32_t d = 0; d < num_pdfs; ++d) nonempty += count[d] > 0;
        auto allot = [&](int64_t target, std::vector<int64_t>* pieces) {
            pieces->assign(num_pdfs, 0);
            using Item = std::pair<double, int32_t>;  // (arcs per piece, pdf)
            std::priority_queue<Item> longest;
            int64_t left = target;
            for (int32_t d = 0; d < num_pdfs; ++d)
                if (count[d] > 0) {
                    (*pieces)[d] = 1;
                    --left;
                    longest.push(Item((double)count[d], d));
                }
            while (left > 0 && !longest.empty()) {
                const int32_t d = longest.top().second;
                longest.pop();
                if ((*pieces)[d] >= count[d]) continue;  // one arc per piece already
                ++(*pieces)[d];
                --left;
                longest.push(Item((double)count[d] / (double)(*pieces)[d], d));
            }
        };
        auto lengths_of = [&](const std::vector<int64_t>& pieces, std::vector<int32_t>* len,
                              std::vector<int32_t>* pdf_of) {
            len->clear();
            pdf_of->clear();
            for (int32_t d = 0; d < num_pdfs; ++d)
                for (int64_t i = 0; i < pieces[d]; ++i) {
                    const int64_t base = count[d] / pieces[d], extra = count[d] % pieces[d];
                    len->push_back((int32_t)(base + (i < extra ? 1 : 0)));
                    pdf_of->push_back(d);
                }
        };
        std::vector<int64_t> pieces, try_pieces;
        std::vector<int32_t> len, pdf_of;
        {
            const int64_t per_k = (int64_t)waves_o * kLanes;
            const int64_t k_min = std::max<int64_t>(1, (nonempty + per_k - 1) / per_k);
            std::vector<std::pair<int64_t, int32_t>> tried;  // (k, fullest wave)
            int32_t best = -1;
            for (int64_t k = k_min; k < k_min + 12; ++k) {
                allot(k * per_k, &try_pieces);
                lengths_of(try_pieces, &len, &pdf_of);
                const Arrangement t = arrange(len, occ_waves, 0);
                tried.emplace_back(k, t.max_wave_slots);
                if (best < 0 || t.max_wave_slots < best) best = t.max_wave_slots;
                if (k * per_k >= A) break;  // one arc per piece
            }
            int64_t k_pick = k_min;
            for (const auto& t : tried)
                if ((double)t.second <= 1.08 * (double)best) { k_pick = t.first; break; }
            allot(k_pick * per_k, &pieces);
            lengths_of(pieces, &len, &pdf_of);
        }
        std::vector<int64_t> first_row(num_pdfs + 1, 0);
        for (int32_t d = 0; d < num_pdfs; ++d) first_row[d + 1] = first_row[d] + pieces[d];
        const int64_t R = first_row[num_pdfs];
        if (R > (int64_t)1 << 28) return "too many occupancy rows";
        const Arrangement ao = arrange(len, occ_waves, 0);
        start_ordering(ao, (int32_t)R, &out->ord[2]);
        out->pdf_first.assign((size_t)num_pdfs + 1, 0);
        out->row_slot.assign((size_t)ao.num_slices * kLanes, -1);
        for (int32_t d = 0; d <= num_pdfs; ++d) out->pdf_first[d] = (int32_t)first_row[d];
        // pdfs cut into many rows: listed after the offsets, for the kernels to add
        // their row sums with a whole wave instead of one thread
        {
            std::vector<int32_t> heavy;
            for (int32_t d = 0; d < num_pdfs; ++d)
                if (pieces[d] > kHeavyPdfRows) heavy.push_back(d);
            out->pdf_first.push_back((int32_t)heavy.size());
            out->pdf_first.push_back(kHeavyPdfRows);
            out->pdf_first.insert(out->pdf_first.end(), heavy.begin(), heavy.end());
        }
        for (int64_t r = 0; r < R; ++r) {
            out->ord[2].row_id[ao.pos[r]] = pdf_of[r];
            out->row_slot[ao.pos[r]] = (int32_t)r;
        }
        {  // padding rows: the words after the last pdf's
            int32_t next = (int32_t)R;
            for (int32_t& q : out->row_slot)
                if (q < 0) q = next++;
        }
        std::vector<int64_t> seen(num_pdfs, 0);
        std::vector<int32_t> prow(A), nth(A), wo(ao.num_slices);
        std::vector<int32_t> bx(A), by(A);  // the words the two gathers read
        for (int64_t a = 0; a < A; ++a) {
            const int32_t d = g.pdf[a];
            // the first `extra` pieces of a pdf hold base + 1 arcs, the others base
            const int64_t base = count[d] / pieces[d], extra = count[d] % pieces[d];
            const int64_t n = seen[d]++, head = extra * (base + 1);
            const int64_t r = first_row[d] + (n < head ? n / (base + 1) : extra + (n - head) / base);
            nth[a] = (int32_t)(n < head ? n % (base + 1) : (n - head) % base);
            prow[a] = ao.pos[r];
            bx[a] = af.pos[g.src[a]];
            by[a] = ab.pos[g.dst[a]];
        }
        for (int32_t sl = 0; sl < ao.num_slices; ++sl) wo[sl] = ao.slice_width[sl];
        const int32_t rf = af.num_slices * kLanes, rb = ab.num_slices * kLanes;
        auto fill = [&](const std::vector<int32_t>& rows, const std::vector<int32_t>& slots,
                        Ordering* o) {
            for (int64_t a = 0; a < A; ++a)
                put(o, rows[a], slots[a], (uint32_t)af.pos[g.src[a]], (uint32_t)ab.pos[g.dst[a]],
                    w[a]);
            if (tune.order_slots) retarget_padding(o, true, false, rf, rb);
        };
        if (tune.order_slots && tune.deal_occ && A >= kDealMinArcs) {
            // two ways to place the arcs; the one whose gathers the bank model prices
            // lower stays: the slots of each row ordered with the rows as they are, or
            // rows and slots dealt together (arcs of a pdf may sit in any of its rows)
            Ordering dealt = out->ord[2];
            std::vector<int32_t> prow_d(prow), nth_d(nth);
            order_slots(prow, bx, by, ao.num_slices, wo, &nth);
            fill(prow, nth, &out->ord[2]);
            deal_occ_arcs(g, pdf_of, len, ao, af.pos, ab.pos, &prow_d, &nth_d);
            fill(prow_d, nth_d, &dealt);
            if (gather_cycles(dealt, true) < gather_cycles(out->ord[2], true))
                out->ord[2] = std::move(dealt);
        } else {
            if (tune.order_slots) order_slots(prow, bx, by, ao.num_slices, wo, &nth);
            fill(prow, nth, &out->ord[2]);
        }
    }
    if (tune.order_slots) {
        const int32_t rf = af.num_slices * kLanes, rb = ab.num_slices * kLanes;
        retarget_padding(&out->ord[0], tune.emission_conflicts, closing != 0, rf, num_pdfs);
        retarget_padding(&out->ord[1], tune.emission_conflicts, closing != 0, rb, num_pdfs);
    }
    out->ord[0].gather_cycles = gather_cycles(out->ord[0], tune.emission_conflicts);
    out->ord[1].gather_cycles = gather_cycles(out->ord[1], tune.emission_conflicts);
    out->ord[2].gather_cycles = gather_cycles(out->ord[2], true);
    return std::string();
}

}  // namespace lfmmi
