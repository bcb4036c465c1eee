// Host-side packing of an HMM graph into sliced-ELL orderings (see pack.h).
#include "pack.h"

#include <algorithm>
#include <cmath>
#include <numeric>

namespace lfmmi {
namespace {

// Where each row goes: rows sorted by length (descending, stable), cut into
// slices of 64, slices dealt to waves longest-first onto the least loaded wave,
// then renumbered so that a wave's slices are consecutive.
struct Arrangement {
    std::vector<int32_t> pos;  // row -> slice * 64 + lane
    std::vector<int32_t> slice_width;
    std::vector<int32_t> wave_first;
    int32_t num_slices = 0, num_waves = 0, max_wave_slots = 0;
};

Arrangement arrange(const std::vector<int32_t>& len, int waves, int extra_slots)
{
    Arrangement ar;
    const int32_t R = (int32_t)len.size();
    ar.num_slices = (R + kLanes - 1) / kLanes;
    ar.num_waves = std::max(1, std::min(waves, ar.num_slices));
    std::vector<int32_t> idx(R);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(),
                     [&](int32_t a, int32_t b) { return len[a] > len[b]; });
    std::vector<int32_t> sorted_width(ar.num_slices);
    for (int32_t s = 0; s < ar.num_slices; ++s)
        sorted_width[s] = len[idx[(size_t)s * kLanes]] + extra_slots;

    std::vector<std::vector<int32_t>> owned(ar.num_waves);
    std::vector<int64_t> load(ar.num_waves, 0);
    for (int32_t s = 0; s < ar.num_slices; ++s) {
        int best = 0;
        for (int w = 1; w < ar.num_waves; ++w)
            if (load[w] < load[best] ||
                (load[w] == load[best] && owned[w].size() < owned[best].size()))
                best = w;
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
    ar.wave_first.assign(ar.num_waves + 1, 0);
    int32_t next = 0;
    for (int w = 0; w < ar.num_waves; ++w) {
        ar.wave_first[w] = next;
        for (int32_t s : owned[w]) {
            for (int l = 0; l < kLanes; ++l) {
                size_t i = (size_t)s * kLanes + l;
                if (i < (size_t)R) ar.pos[idx[i]] = next * kLanes + l;
            }
            ar.slice_width.push_back(sorted_width[s]);
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

}  // namespace

int choose_waves(int64_t num_arcs, int32_t num_states)
{
    // about 8 arc slots per lane before a further wave pays for its share of
    // the per-frame barriers; never more waves than slices of states
    int64_t by_arcs = (num_arcs + (int64_t)kLanes * 8 - 1) / ((int64_t)kLanes * 8);
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
                       bool per_arc_leak, PackedGraph* out, bool* bad_graph)
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
    const Arrangement af = arrange(indeg, rec_waves, 1);
    const Arrangement ab = arrange(outdeg, rec_waves, 1);
    if (af.num_slices * kLanes > kMaxIndex) return "too many states";
    start_ordering(af, S, &out->ord[0]);
    start_ordering(ab, S, &out->ord[1]);
    for (int32_t s = 0; s < S; ++s) {
        out->ord[0].row_id[af.pos[s]] = s;
        out->ord[1].row_id[ab.pos[s]] = s;
    }
    std::vector<float> w(A);
    for (int64_t a = 0; a < A; ++a) w[a] = (float)std::exp((double)g.logw[a]);
    {
        std::vector<int32_t> nf(S, 0), nb(S, 0);
        for (int64_t a = 0; a < A; ++a) {
            const int32_t i = g.src[a], j = g.dst[a];
            put(&out->ord[0], af.pos[j], nf[j]++, (uint32_t)af.pos[i], (uint32_t)g.pdf[a], w[a]);
            put(&out->ord[1], ab.pos[i], nb[i]++, (uint32_t)ab.pos[j], (uint32_t)g.pdf[a], w[a]);
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
        for (int32_t sl = 0; sl < o.num_slices; ++sl)
            for (int l = 0; l < kLanes; ++l) {
                const size_t at = (size_t)(o.slice_off[sl + 1] - 1) * kLanes + l;
                o.key[at] = 0u;
                o.w[at] = out->va[d][(size_t)sl * kLanes + l];
            }
        o.wave_mask.assign(o.num_waves, 0);
        for (int32_t wv = 0; wv < o.num_waves; ++wv) {
            const int32_t first = o.slice_off[o.wave_first[wv]];
            const int32_t count = o.slice_off[o.wave_first[wv + 1]] - first;
            if (count > 64) continue;
            for (int32_t sl = o.wave_first[wv]; sl < o.wave_first[wv + 1]; ++sl)
                o.wave_mask[wv] |= (uint64_t)1 << (o.slice_off[sl + 1] - 1 - first);
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
            std::vector<int32_t> nf(S, 0), nb(S, 0);
            for (int64_t a = 0; a < A; ++a) {
                const int32_t i = g.src[a], j = g.dst[a];
                const int32_t pf = af.pos[j], pb = ab.pos[i];
                of.wb[(size_t)(of.slice_off[pf / kLanes] + nf[j]++) * kLanes + pf % kLanes] =
                    w[a] * g.init_prob[i];
                ob.wb[(size_t)(ob.slice_off[pb / kLanes] + nb[i]++) * kLanes + pb % kLanes] = w[a];
            }
        }
    }

    // ---- OCC: arcs grouped by pdf, each pdf's list cut into pieces
    {
        const int lanes_total = kLanes * std::max(1, occ_waves);
        int64_t piece = (A + lanes_total - 1) / lanes_total;
        piece = std::max<int64_t>(4, std::min<int64_t>(piece, 32));
        std::vector<int64_t> count(num_pdfs, 0);
        for (int64_t a = 0; a < A; ++a) ++count[g.pdf[a]];
        std::vector<int64_t> first_row(num_pdfs + 1, 0);
        for (int32_t d = 0; d < num_pdfs; ++d)
            first_row[d + 1] = first_row[d] + (count[d] + piece - 1) / piece;
        const int64_t R = first_row[num_pdfs];
        if (R > (int64_t)1 << 28) return "too many occupancy rows";
        std::vector<int32_t> len((size_t)R, 0), pdf_of((size_t)R, 0);
        for (int32_t d = 0; d < num_pdfs; ++d)
            for (int64_t r = first_row[d], left = count[d]; r < first_row[d + 1]; ++r) {
                len[r] = (int32_t)std::min<int64_t>(piece, left);
                left -= len[r];
                pdf_of[r] = d;
            }
        const Arrangement ao = arrange(len, occ_waves, 0);
        start_ordering(ao, (int32_t)R, &out->ord[2]);
        out->row_pdf4.assign((size_t)ao.num_slices * kLanes, -1);
        for (int64_t r = 0; r < R; ++r) {
            out->ord[2].row_id[ao.pos[r]] = pdf_of[r];
            out->row_pdf4[ao.pos[r]] = pdf_of[r] * 4;
        }
        std::vector<int64_t> seen(num_pdfs, 0);
        for (int64_t a = 0; a < A; ++a) {
            const int32_t d = g.pdf[a];
            const int64_t r = first_row[d] + seen[d] / piece;
            const int32_t nth = (int32_t)(seen[d] % piece);
            ++seen[d];
            put(&out->ord[2], ao.pos[r], nth, (uint32_t)af.pos[g.src[a]],
                (uint32_t)ab.pos[g.dst[a]], w[a]);
        }
    }
    return std::string();
}

}  // namespace lfmmi
