// Host-side graph packing: three sliced-ELL (64 rows per slice) arc orderings.
//
// Section 3.3 keeps the transition list twice, sorted by from-state and by
// to-state, each with per-state index ranges. The same information is kept here
// as three orderings whose rows are owned by lanes of a wavefront:
//   FWD  rows = to-states    record (from-state, pdf)      alpha recursion
//   BWD  rows = from-states  record (to-state, pdf)        beta recursion
//   OCC  rows = pieces of a pdf-id's arc list, record (from-state, to-state)
//        pdf occupancies of Eq. 3
// Rows are sorted by length so that the 64 rows of a slice are padded little,
// slices are dealt to the waves of a workgroup by longest-processing-time, and
// states are renumbered per ordering so that the row a lane owns is
// slice * 64 + lane (coalesced trellis rows, conflict-free owner accesses).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace lfmmi {

constexpr int kLanes = 64;
constexpr int kHeavyPdfRows = 24;  // OCC: more rows than this and a wave adds them up
constexpr int kMaxWaves = 16;
constexpr int kMaxIndex = 16384;  // x / y index * 4 must fit 16 bits

struct Ordering {
    int32_t num_rows = 0;        // real rows
    int32_t num_slices = 0;      // rows padded to kLanes
    int32_t num_waves = 0;       // waves that own slices
    int32_t total_slots = 0;     // sum of slice widths
    int32_t max_wave_slots = 0;  // largest per-wave sum of widths
    std::vector<int32_t> slice_off;   // [num_slices + 1]
    std::vector<int32_t> wave_first;  // [num_waves + 1]
    std::vector<uint32_t> key;        // [total_slots * 64]
    std::vector<float> w;             // [total_slots * 64]
    std::vector<float> wb;            // non-uniform pi only: FWD w * pi[from-state], BWD w
    std::vector<int32_t> row_id;      // [num_slices * 64], -1 = padding row
    // FWD / BWD only. closing_slots: every slice ends in one extra slot that holds
    // no arc but the row's leak-dot weight a[row] (FWD 1, BWD pi[row], 0 on padding
    // rows); packed so when pi is not uniform. Otherwise a[row] is the constant
    // a_const on every real row and slices hold arcs (and padding) only.
    // wave_mask[w] has bit i set when slot i of wave w is the last of a slice
    // (0 when the wave owns more than 64 slots).
    int32_t closing_slots = 0;
    float a_const = 0.f;
    std::vector<uint64_t> wave_mask;  // [num_waves]
    // Hub slices (FWD / BWD): slice_hub[s] != 0 when the 64 lanes of slice s all hold
    // arcs of the row of lane 0 (a row with far more arcs than the others); its
    // other 63 rows are padding rows. wave_hub[w]: the bits of wave_mask[w] that
    // belong to hub slices.
    std::vector<int32_t> slice_hub;   // [num_slices]
    std::vector<uint64_t> wave_hub;   // [num_waves]
    int64_t gather_cycles = 0;        // modelled LDS cycles of the gathers of one frame
    float b_const = 0.f;              // leak target when it is one constant (BWD 1, FWD uniform pi)
    int32_t has_wb = 0;               // wb is filled
};

struct PackedGraph {
    int32_t num_states = 0;
    int64_t num_arcs = 0;
    Ordering ord[3];
    // Per-direction vectors in that direction's row numbering, padded with 0:
    //   init: start vector (FWD pi, BWD final)      fin: closing dot (FWD final, BWD pi)
    //   a:    leak dot weights (FWD 1, BWD pi)      b:   leak target (FWD pi, BWD 1)
    std::vector<float> vinit[2], va[2], vb[2], vfin[2];
    // Emission by entered state: true when all arcs into a state carry one pdf-id
    // (graphs expanded from HMMs whose states emit, Section 4.2: the emission of an
    // arc is then a function of its to-state). row_pdf[d][row]: that pdf-id for the
    // state that owns the row in direction d's numbering (0 on padding rows and for
    // states nothing enters); filled only when the flag is set.
    bool pdf_by_dst = false;
    std::vector<int32_t> row_pdf[2];
    // OCC: a frame's row sums are stored sorted by pdf: the sum of row position
    // slice * 64 + lane is word row_slot[position]; pdf d owns words pdf_first[d] ..
    // pdf_first[d + 1] - 1, added up in that order (padding rows: the words after)
    // then: the number H of pdfs with more than kHeavyPdfRows rows, that limit,
    // and the H pdf-ids (ascending)
    std::vector<int32_t> pdf_first;  // [num_pdfs + 1] + [2 + H]
    std::vector<int32_t> row_slot;   // [OCC num_slices * 64], a permutation
};

struct ArcList {
    int32_t num_states;
    int64_t num_arcs;
    const int32_t* src;
    const int32_t* dst;
    const int32_t* pdf;
    const float* logw;
    const float* init_prob;
    const float* final_prob;
};

// Waves per workgroup that suit a graph with this many arcs.
int choose_waves(int64_t num_arcs, int32_t num_states);

// Validates and packs one graph. Returns an empty string on success, else the
// reason (bad_graph says whether the graph or an argument is at fault).
// What the packer does about LDS bank conflicts of the fp32 kernels.
struct PackTuning {
    bool balance_banks = true;        // re-deal lanes inside half-slices (state -> bank)
    bool order_slots = true;          // order each row's arcs over its slots
    bool emission_conflicts = true;   // the emission gather can conflict (row not replicated)
    bool hub_slices = true;           // rows with far more arcs than the others get a slice each
    bool deal_occ = true;             // OCC ordering: arcs dealt to rows and slots jointly
};

// per_arc_leak: fill the per-arc leak factors (required when init_prob is not
// uniform over the states).
std::string pack_graph(const ArcList& g, int32_t num_pdfs, int rec_waves, int occ_waves,
                       bool per_arc_leak, const PackTuning& tune, PackedGraph* out,
                       bool* bad_graph);
// True when every state has the same initial probability.
bool uniform_init(const ArcList& g);

}  // namespace lfmmi
