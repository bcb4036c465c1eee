// C ABI of the LF-MMI forward-backward library: handle management, argument
// checks, workspace layout and kernel launches. See include/lfmmi.h.
#include "../../include/lfmmi.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <string>
#include <thread>
#include <vector>

#include "kernels.h"
#include "pack.h"

using namespace lfmmi;

static_assert(LFMMI_STATIC_WORKSPACE_BYTES == kStaticWorkspaceBytes &&
                  LFMMI_STATIC_MAX_BATCH == kStaticMaxBatch,
              "the header states the limits of the static workspace");

namespace {

thread_local std::string g_error;

lfmmi_status fail(lfmmi_status st, const std::string& msg)
{
    g_error = msg;
    return st;
}

lfmmi_status fail_hip(hipError_t e, const char* what)
{
    return fail(LFMMI_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

constexpr size_t kLdsBytes = 160 * 1024;
constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int env_int(const char* name, int fallback)
{
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

}  // namespace

struct lfmmi_graph {
    int32_t num_graphs = 0;
    int32_t num_pdfs = 0;
    int64_t total_states = 0, total_arcs = 0;
    int rec_waves = 1, occ_waves = 1;
    std::vector<PackedGraph> packed;
    std::vector<OrdDesc> ords;  // [num_graphs * 3]
    int32_t max_rows_f = 0, max_rows_b = 0, max_rows_occ = 0;
    bool wide = false;  // fp64 state vectors (some state is not final)
    int rec_nslot = 0;  // register-resident arc slots of the recursion kernel (0: streamed)
    bool rec_yrep = false;
    bool rec_hubs = false;  // some FWD / BWD ordering has hub slices
    int rec_hybrid = 0;  // 1, 2: rec_nslot slots of a wave in registers, its others streamed
                         // (2: LDS map for up to 12288 states)
    bool has_wb = false;  // arcs carry a per-arc leak factor (some init_prob is not uniform)
    bool rec_grouped = false;  // every arc takes the pdf of the state it enters and the
                               // recursion runs the variant without an emission gather

    // device copy
    bool uploaded = false;
    int device = -1;
    void* dev_base = nullptr;
    DeviceGraph dg{};

    // workspace, grown on demand
    void* ws = nullptr;
    size_t ws_bytes = 0;
    // lengths and T of the call whose descriptors the workspace holds (empty: none)
    std::vector<int32_t> desc_lengths;
    int32_t desc_T = -1;
    // pinned staging for per-call descriptors
    void* stage = nullptr;
    size_t stage_bytes = 0;
    hipEvent_t stage_done = nullptr;
    bool stage_pending = false;

    // emission values of the last call on this handle (inside ws), for the pass that
    // follows it in a full-loss call; and values borrowed from the other handle
    float* last_emis = nullptr;
    float* last_rowmax = nullptr;
    size_t last_emis_count = 0;  // B * T * P of that call
    const float* borrow_emis = nullptr;
    const float* borrow_rowmax = nullptr;

    // streams and events of the concurrent buckets of a call, made on first use
    hipEvent_t fork = nullptr;
    hipEvent_t join[Buckets::kMax] = {nullptr, nullptr, nullptr, nullptr};  // [0] unused

    // profiling: per call made while enabled 4 * (its bucket count) events
    int profile = 0;  // 0 off, 1 events around every kernel, 2 around the recursion only
    std::vector<hipEvent_t> ev;
    std::vector<int32_t> ev_buckets;  // bucket count of each profiled call
    std::vector<hipEvent_t> ev_free;  // events of calls already read, used again
};

namespace {

lfmmi_status pack_all(int32_t n, int32_t num_pdfs, const int64_t* state_off,
                      const int64_t* arc_off, const int32_t* src, const int32_t* dst,
                      const int32_t* pdf, const float* logw, const float* init_prob,
                      const float* final_prob, lfmmi_graph** out)
{
    if (!out) return fail(LFMMI_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (n < 1) return fail(LFMMI_ERR_INVALID_ARG, "number of graphs must be >= 1");
    if (num_pdfs < 1) return fail(LFMMI_ERR_INVALID_ARG, "num_pdfs must be >= 1");
    if (num_pdfs > kMaxIndex)
        return fail(LFMMI_ERR_UNSUPPORTED, "num_pdfs exceeds 16384");
    if (!state_off || !arc_off) return fail(LFMMI_ERR_INVALID_ARG, "null offset array");
    if (state_off[0] != 0 || arc_off[0] != 0)
        return fail(LFMMI_ERR_INVALID_ARG, "offsets must start at 0");
    for (int32_t g = 0; g < n; ++g) {
        if (state_off[g + 1] - state_off[g] < 1)
            return fail(LFMMI_ERR_INVALID_ARG, "graph " + std::to_string(g) + " has no state");
        if (state_off[g + 1] - state_off[g] > kMaxIndex)
            return fail(LFMMI_ERR_UNSUPPORTED,
                        "graph " + std::to_string(g) + " has more than 16384 states");
        if (arc_off[g + 1] < arc_off[g])
            return fail(LFMMI_ERR_INVALID_ARG, "arc offsets must not decrease");
    }
    lfmmi_graph* h = new (std::nothrow) lfmmi_graph();
    if (!h) return fail(LFMMI_ERR_OOM, "host allocation failed");
    try {
        h->num_graphs = n;
        h->num_pdfs = num_pdfs;
        h->total_states = state_off[n];
        h->total_arcs = arc_off[n];
        // fp32 state vectors when every state is both initial and final: a leak then
        // feeds every state of alpha and of beta a share of the frame's total, which
        // bounds how far below that total a state that carries posterior mass can
        // sit, and fp32 holds it. Otherwise (left-to-right graphs: a numerator, or any
        // graph entered through one state) that mass can sit tens of orders of
        // magnitude below the total: fp64. (With leak = 0 nothing bounds it in an fp32
        // graph either; the scan then flags a sequence whose two passes disagree.)
        bool all_final = true, all_initial = true;
        if (final_prob)
            for (int64_t s = 0; s < state_off[n]; ++s) all_final = all_final && final_prob[s] > 0.f;
        if (init_prob)
            for (int64_t s = 0; s < state_off[n]; ++s) all_initial = all_initial && init_prob[s] > 0.f;
        h->wide = !(all_final && all_initial);
        if (const char* v = std::getenv("LFMMI_PRECISION")) {
            if (std::atoi(v) == 64) h->wide = true;
            if (std::atoi(v) == 32) h->wide = false;
        }
        auto arcs_of = [&](int32_t g) {
            ArcList al;
            al.num_states = (int32_t)(state_off[g + 1] - state_off[g]);
            al.num_arcs = arc_off[g + 1] - arc_off[g];
            al.src = src ? src + arc_off[g] : nullptr;
            al.dst = dst ? dst + arc_off[g] : nullptr;
            al.pdf = pdf ? pdf + arc_off[g] : nullptr;
            al.logw = logw ? logw + arc_off[g] : nullptr;
            al.init_prob = init_prob ? init_prob + state_off[g] : nullptr;
            al.final_prob = final_prob ? final_prob + state_off[g] : nullptr;
            return al;
        };
        h->has_wb = false;
        if (init_prob)
            for (int32_t g = 0; g < n; ++g) h->has_wb = h->has_wb || !uniform_init(arcs_of(g));

        // the emission row is replicated once per LDS bank when it is small
        {
            int64_t max_states = 0;
            for (int32_t g = 0; g < n; ++g)
                max_states = std::max(max_states, state_off[g + 1] - state_off[g]);
            const int rows_guess = (int)((max_states + kLanes - 1) / kLanes * kLanes);
            h->rec_yrep = num_pdfs <= 255 &&
                          rec_lds_bytes(rows_guess, num_pdfs, h->wide, true) <= 96 * 1024;
            if (env_int("LFMMI_YREP", 1) == 0) h->rec_yrep = false;
        }
        PackTuning tune;
        tune.emission_conflicts = !h->rec_yrep;
        tune.balance_banks = !h->wide && env_int("LFMMI_BALANCE", 1) != 0;
        tune.order_slots = !h->wide && env_int("LFMMI_ORDER", 1) != 0;
        tune.hub_slices = env_int("LFMMI_HUBS", 1) != 0;
        tune.deal_occ = env_int("LFMMI_DEAL", 1) != 0;

        int waves = 1;
        for (int32_t g = 0; g < n; ++g)
            waves = std::max(waves, choose_waves(arc_off[g + 1] - arc_off[g],
                                                 (int32_t)(state_off[g + 1] - state_off[g])));
        const int forced = env_int("LFMMI_WAVES", 0);
        if (forced > 0) waves = std::min(forced, kMaxWaves);
        // Pack for `waves` waves; when the arcs of a wave then fit no register-resident
        // variant of the recursion kernel, try half the waves (twice the registers per
        // lane) before settling for streamed arcs.
        // (called once the graphs are packed: what has to fit the fixed LDS map of
        // those kernels, 32 KB per state vector, is the padded row count of the
        // orderings - hub slices add 63 padding rows each - not the state count;
        // it does not depend on the number of waves)
        auto registers_possible = [&](int wv) {
            if (h->rec_yrep ? num_pdfs > 255 : num_pdfs > 3072) return false;  // staging limits
            if (std::max(h->max_rows_f, h->max_rows_b) > (h->wide ? 4096 : 8192)) return false;
            for (int32_t g = 0; g < n; ++g)
                if ((double)(arc_off[g + 1] - arc_off[g]) / (64.0 * wv) > 48.0) return false;
            return true;
        };
        auto pack_with = [&](int wv, int* max_slots) -> lfmmi_status {
            h->rec_waves = wv;
            // the occupancy pass is throughput work: about 8 arcs per lane, at most 8 waves
            int64_t most_arcs = 0;
            for (int32_t g = 0; g < n; ++g) most_arcs = std::max(most_arcs, arc_off[g + 1] - arc_off[g]);
            const int by_arcs = (int)std::max<int64_t>(1, (most_arcs + 511) / 512);
            // (16 where the states allow one frame per arc record only: its kernel
            // keeps more loads in flight with more waves)
            int64_t most_states = 0;
            for (int32_t g = 0; g < n; ++g)
                most_states = std::max(most_states, state_off[g + 1] - state_off[g]);
            const int cap = !h->wide && most_states * 4 > 16384 ? 16 : 8;
            h->occ_waves = std::min(by_arcs, env_int("LFMMI_OCC_WAVES", cap));
            h->packed.assign(n, PackedGraph());
            h->max_rows_f = h->max_rows_b = h->max_rows_occ = 0;
            h->rec_hubs = false;
            *max_slots = 0;
            // the graphs of a batch are packed independently: on several threads
            std::vector<std::string> errs(n);
            std::vector<char> bads(n, 0);
            {
                const unsigned hw = std::max(1u, std::thread::hardware_concurrency());
                const int workers = (int)std::max(1u, std::min({hw, 16u, (unsigned)(n / 8 + 1)}));
                std::atomic<int32_t> next(0);
                const int rec_w = h->rec_waves, occ_w = h->occ_waves;
                const bool wb = h->has_wb;
                auto work = [&]() {
                    for (int32_t g = next.fetch_add(1); g < n; g = next.fetch_add(1)) {
                        bool bad = false;
                        try {
                            errs[g] = pack_graph(arcs_of(g), num_pdfs, rec_w, occ_w, wb, tune,
                                                 &h->packed[g], &bad);
                        } catch (const std::bad_alloc&) {
                            errs[g] = "host allocation failed";
                        }
                        bads[g] = bad ? 1 : 0;
                    }
                };
                std::vector<std::thread> pool;
                for (int t = 1; t < workers; ++t) pool.emplace_back(work);
                work();
                for (std::thread& t : pool) t.join();
            }
            for (int32_t g = 0; g < n; ++g) {
                if (!errs[g].empty())
                    return fail(bads[g] ? LFMMI_ERR_BAD_GRAPH : LFMMI_ERR_INVALID_ARG,
                                (n > 1 ? "graph " + std::to_string(g) + ": " : std::string()) + errs[g]);
                h->max_rows_f = std::max(h->max_rows_f, h->packed[g].ord[0].num_slices * kLanes);
                h->max_rows_b = std::max(h->max_rows_b, h->packed[g].ord[1].num_slices * kLanes);
                h->max_rows_occ = std::max(h->max_rows_occ, h->packed[g].ord[2].num_slices * kLanes);
                for (int o = 0; o < 2; ++o) {
                    *max_slots = std::max(*max_slots, h->packed[g].ord[o].max_wave_slots);
                    for (int32_t f : h->packed[g].ord[o].slice_hub) h->rec_hubs = h->rec_hubs || f != 0;
                }
            }
            return LFMMI_OK;
        };
        {
            int max_slots = 0;
            lfmmi_status st = pack_with(waves, &max_slots);
            // the replicated emission row was granted on the state count; with the padded
            // rows known it is given up when the two no longer fit LDS together (the
            // slot order then ignores emission conflicts: slower, never wrong)
            if (st == LFMMI_OK && h->rec_yrep &&
                rec_lds_bytes(std::max(h->max_rows_f, h->max_rows_b), num_pdfs, h->wide, true) > kLdsBytes)
                h->rec_yrep = false;
            // Graphs whose arcs all take the pdf of the state they enter: the variant
            // without an emission gather, when every wave's arcs fit its registers
            // (two per slot), the workgroup's threads can stage an emission value per row
            // in the passes that variant has, and the rows leave the last slice of the
            // LDS map to the zero word.
            // It pays from about a dozen slots per wave on: what it saves grows with the
            // arcs, what beta's second barrier costs does not (the 128 numerator graphs
            // of the e2e workload, 4 slots per wave: 366 us with it, 314 us without).
            // LFMMI_GROUPED=0 never takes it, 2 takes it whenever it applies.
            auto grouped_slots = [&]() {
                const int want = env_int("LFMMI_GROUPED", 1);
                if (want == 0 || h->rec_hubs) return 0;
                if (want != 2 && max_slots < 16) return 0;
                const int rows_most = std::max(h->max_rows_f, h->max_rows_b);
                if (rows_most > (h->wide ? 4096 : 8192) - kLanes) return 0;
                if (rows_most > rec_grouped_max_rows(waves * kLanes)) return 0;
                for (int32_t g = 0; g < n; ++g)
                    if (!h->packed[g].pdf_by_dst) return 0;
                return rec_grouped_slots(h->wide, h->has_wb, max_slots, waves * kLanes);
            };
            const int gslots = st == LFMMI_OK ? grouped_slots() : 0;
            h->rec_grouped = gslots > 0;
            auto resident = [&](int slots, int wv) {
                return rec_register_slots(h->wide, h->has_wb, h->rec_yrep, h->rec_hubs, slots,
                                          wv * kLanes);
            };
            // too many arcs for the registers: keep the first slots of every wave there
            // and stream the others, where the fixed LDS map of that kernel holds the graph
            auto hybrid_possible = [&]() {  // 0: no; 1: 32 KB state vectors; 2: 48 KB
                if (h->wide || h->has_wb || env_int("LFMMI_HYBRID", 1) == 0) return 0;
                if (h->rec_yrep ? num_pdfs > 255 : num_pdfs > 3072) return 0;
                // padded rows, not states: see registers_possible
                const int most = std::max(h->max_rows_f, h->max_rows_b);
                const int map = most <= 8192 ? 1 : (most <= 12288 && !h->rec_yrep ? 2 : 0);
                return map != 0 && rec_hybrid_slots(h->wide, h->has_wb, h->rec_yrep, h->rec_hubs,
                                                    map) > 0
                           ? map
                           : 0;
            };
            // Not every combination of slot count, replicated emission row and hub code
            // is built (some would spill registers): when nothing fits with the
            // replicated row, the choice is made again with plain emission rows.
            for (int attempt = 0; attempt < 2 && st == LFMMI_OK; ++attempt) {
                h->rec_nslot = gslots > 0 ? gslots
                               : registers_possible(waves) ? resident(max_slots, waves)
                                                           : 0;
                if (h->rec_nslot == 0 && !h->wide && forced <= 0 && waves > 8 &&
                    registers_possible(waves / 2) && resident(2 * max_slots, waves / 2) != 0) {
                    waves /= 2;
                    st = pack_with(waves, &max_slots);
                    h->rec_nslot = st == LFMMI_OK ? resident(max_slots, waves) : 0;
                }
                if (st == LFMMI_OK && h->rec_nslot == 0 && hybrid_possible() != 0) {
                    h->rec_hybrid = hybrid_possible();
                    h->rec_nslot = rec_hybrid_slots(h->wide, h->has_wb, h->rec_yrep, h->rec_hubs,
                                                    h->rec_hybrid);
                }
                if (h->rec_nslot != 0 || !h->rec_yrep) break;
                h->rec_yrep = false;
            }
            if (st != LFMMI_OK) {
                delete h;
                return st;
            }
        }
        const int rows = std::max(h->max_rows_f, h->max_rows_b);
        if (rec_lds_bytes(rows, num_pdfs, h->wide, h->rec_yrep) > kLdsBytes ||
            occ_lds_bytes(h->max_rows_f, h->max_rows_b, h->max_rows_occ, h->wide) > kLdsBytes) {
            delete h;
            return fail(LFMMI_ERR_UNSUPPORTED,
                        "states and pdfs do not fit the 160 KB of LDS of one compute unit");
        }
    } catch (const std::bad_alloc&) {
        delete h;
        return fail(LFMMI_ERR_OOM, "host allocation failed");
    }
    *out = h;
    return LFMMI_OK;
}

template <class T>
size_t reserve(size_t* total, size_t count)
{
    const size_t at = *total;
    *total = align_up(at + count * sizeof(T));
    return at;
}

lfmmi_status upload(lfmmi_graph* h)
{
    if (h->uploaded) return LFMMI_OK;
    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    {
        // once per device and process: the LDS limits of every kernel variant
        static std::mutex mu;
        static std::vector<int> done;
        std::lock_guard<std::mutex> lock(mu);
        if (std::find(done.begin(), done.end(), h->device) == done.end()) {
            if ((e = configure_kernels()) != hipSuccess) return fail_hip(e, "hipFuncSetAttribute");
            // ... and the address of this device's copy of the static workspace
            if ((e = find_static_workspace(h->device)) != hipSuccess)
                return fail_hip(e, "hipGetSymbolAddress");
            done.push_back(h->device);
        }
    }

    // concatenate every graph's orderings
    size_t n_slots = 0, n_soff = 0, n_wf = 0, n_vec = 0, n_rowpdf = 0, n_mask = 0, n_pfirst = 0;
    h->ords.assign((size_t)h->num_graphs * 3, OrdDesc{});
    for (int32_t g = 0; g < h->num_graphs; ++g)
        for (int o = 0; o < 3; ++o) {
            const Ordering& od = h->packed[g].ord[o];
            OrdDesc& d = h->ords[(size_t)g * 3 + o];
            d.num_slices = od.num_slices;
            d.num_waves = od.num_waves;
            d.rec_at = (int32_t)n_slots;
            d.slice_off_at = (int32_t)n_soff;
            d.wave_first_at = (int32_t)n_wf;
            d.max_wave_slots = od.max_wave_slots;
            d.total_slots = od.total_slots;
            d.mask_at = (int32_t)n_mask;
            d.has_wb = od.has_wb;
            d.b_const = od.b_const;
            d.closing = od.closing_slots;
            d.a_const = od.a_const;
            n_mask += od.wave_mask.size();
            n_slots += od.total_slots;
            n_soff += od.slice_off.size();
            n_wf += od.wave_first.size();
            if (o < 2) {
                // FWD and BWD vectors of one graph sit back to back
                d.vec_at = (int32_t)n_vec;
                n_vec += (size_t)od.num_slices * kLanes;
            } else {
                d.vec_at = (int32_t)n_rowpdf;
                n_rowpdf += (size_t)od.num_slices * kLanes;
                d.pdf_first_at = (int32_t)n_pfirst;
                n_pfirst += h->packed[g].pdf_first.size();
            }
        }
    if (n_slots > (size_t)1 << 30) return fail(LFMMI_ERR_UNSUPPORTED, "packed graph too large");
    for (const OrdDesc& d : h->ords)
        if (d.total_slots % 2 != 0) return fail(LFMMI_ERR_INVALID_ARG, "odd slot count (packer)");

    size_t total = 0;
    const size_t at_recs = reserve<uint2>(&total, n_slots * kLanes);
    const size_t at_wb = reserve<float>(&total, n_slots * kLanes);
    const size_t at_mask = reserve<uint64_t>(&total, n_mask);
    const size_t at_hubmask = reserve<uint64_t>(&total, n_mask);
    const size_t at_shub = reserve<int32_t>(&total, n_soff);
    const size_t at_soff = reserve<int32_t>(&total, n_soff);
    const size_t at_wf = reserve<int32_t>(&total, n_wf);
    const size_t at_vinit = reserve<float>(&total, n_vec);
    const size_t at_va = reserve<float>(&total, n_vec);
    const size_t at_vb = reserve<float>(&total, n_vec);
    const size_t at_vfin = reserve<float>(&total, n_vec);
    const size_t at_rowpdfs = reserve<int32_t>(&total, n_vec);
    const size_t at_rowpdf = reserve<int32_t>(&total, n_rowpdf);
    const size_t at_pfirst = reserve<int32_t>(&total, n_pfirst);
    const size_t at_ords = reserve<OrdDesc>(&total, h->ords.size());
    total = std::max<size_t>(total, kAlign);

    std::vector<unsigned char> host;
    try {
        host.assign(total, 0);
    } catch (const std::bad_alloc&) {
        return fail(LFMMI_ERR_OOM, "host allocation failed");
    }
    for (int32_t g = 0; g < h->num_graphs; ++g)
        for (int o = 0; o < 3; ++o) {
            const Ordering& od = h->packed[g].ord[o];
            const OrdDesc& d = h->ords[(size_t)g * 3 + o];
            // On the device the records of slots 2q and 2q + 1 of a lane lie side by
            // side (one 16-byte load), pair q of lane l at [q * 64 + l]; every slice
            // starts at an even slot.
            uint2* recs = reinterpret_cast<uint2*>(host.data() + at_recs) + (size_t)d.rec_at * kLanes;
            float* wbs = reinterpret_cast<float*>(host.data() + at_wb) + (size_t)d.rec_at * kLanes;
            for (size_t i = 0; i < od.key.size(); ++i) {
                const size_t slot = i / kLanes, lane = i % kLanes;
                const size_t to = ((slot >> 1) * kLanes + lane) * 2 + (slot & 1);
                uint32_t wbits;
                std::memcpy(&wbits, &od.w[i], 4);
                uint32_t key = od.key[i];
                // replicated emission rows: the upper half becomes the byte offset of
                // this lane's copy of the value, 128 * pdf + 4 * (lane % 32)
                if (o < 2 && h->rec_yrep)
                    key = (key & 0xffffu) | (((key >> 16) * 32u + (uint32_t)(lane & 31) * 4u) << 16);
                recs[to] = make_uint2(key, wbits);
                if (!od.wb.empty()) wbs[to] = od.wb[i];
            }
            if (!od.wave_mask.empty())
                std::memcpy(host.data() + at_mask + (size_t)d.mask_at * 8, od.wave_mask.data(),
                            od.wave_mask.size() * 8);
            if (!od.wave_hub.empty())
                std::memcpy(host.data() + at_hubmask + (size_t)d.mask_at * 8, od.wave_hub.data(),
                            od.wave_hub.size() * 8);
            if (!od.slice_hub.empty())  // indexed like slice_off (one entry fewer)
                std::memcpy(host.data() + at_shub + (size_t)d.slice_off_at * 4, od.slice_hub.data(),
                            od.slice_hub.size() * 4);
            std::memcpy(host.data() + at_soff + (size_t)d.slice_off_at * 4, od.slice_off.data(),
                        od.slice_off.size() * 4);
            std::memcpy(host.data() + at_wf + (size_t)d.wave_first_at * 4, od.wave_first.data(),
                        od.wave_first.size() * 4);
            const size_t nrow = (size_t)od.num_slices * kLanes;
            if (o < 2) {
                const PackedGraph& pg = h->packed[g];
                std::memcpy(host.data() + at_vinit + (size_t)d.vec_at * 4, pg.vinit[o].data(), nrow * 4);
                std::memcpy(host.data() + at_va + (size_t)d.vec_at * 4, pg.va[o].data(), nrow * 4);
                std::memcpy(host.data() + at_vb + (size_t)d.vec_at * 4, pg.vb[o].data(), nrow * 4);
                std::memcpy(host.data() + at_vfin + (size_t)d.vec_at * 4, pg.vfin[o].data(), nrow * 4);
                if (pg.row_pdf[o].size() == nrow)
                    std::memcpy(host.data() + at_rowpdfs + (size_t)d.vec_at * 4, pg.row_pdf[o].data(),
                                nrow * 4);
            } else {
                const PackedGraph& pg = h->packed[g];
                std::memcpy(host.data() + at_rowpdf + (size_t)d.vec_at * 4, pg.row_slot.data(),
                            nrow * 4);
                std::memcpy(host.data() + at_pfirst + (size_t)d.pdf_first_at * 4,
                            pg.pdf_first.data(), pg.pdf_first.size() * 4);
            }
        }
    std::memcpy(host.data() + at_ords, h->ords.data(), h->ords.size() * sizeof(OrdDesc));

    if ((e = hipMalloc(&h->dev_base, total)) != hipSuccess) {
        h->dev_base = nullptr;
        return fail(LFMMI_ERR_OOM, std::string("hipMalloc: ") + hipGetErrorString(e));
    }
    if ((e = hipMemcpy(h->dev_base, host.data(), total, hipMemcpyHostToDevice)) != hipSuccess) {
        (void)hipFree(h->dev_base);
        h->dev_base = nullptr;
        return fail_hip(e, "hipMemcpy");
    }
    unsigned char* base = static_cast<unsigned char*>(h->dev_base);
    h->dg.recs = reinterpret_cast<const uint2*>(base + at_recs);
    h->dg.wb = reinterpret_cast<const float*>(base + at_wb);
    h->dg.wave_mask = reinterpret_cast<const uint64_t*>(base + at_mask);
    h->dg.wave_hub = reinterpret_cast<const uint64_t*>(base + at_hubmask);
    h->dg.slice_hub = reinterpret_cast<const int32_t*>(base + at_shub);
    h->dg.slice_off = reinterpret_cast<const int32_t*>(base + at_soff);
    h->dg.wave_first = reinterpret_cast<const int32_t*>(base + at_wf);
    h->dg.vinit = reinterpret_cast<const float*>(base + at_vinit);
    h->dg.va = reinterpret_cast<const float*>(base + at_va);
    h->dg.vb = reinterpret_cast<const float*>(base + at_vb);
    h->dg.vfin = reinterpret_cast<const float*>(base + at_vfin);
    h->dg.row_pdf = reinterpret_cast<const int32_t*>(base + at_rowpdfs);
    h->dg.row_slot = reinterpret_cast<const int32_t*>(base + at_rowpdf);
    h->dg.pdf_first = reinterpret_cast<const int32_t*>(base + at_pfirst);
    h->dg.ords = reinterpret_cast<const OrdDesc*>(base + at_ords);
    h->uploaded = true;
    return LFMMI_OK;
}

// Streams of the buckets 1 .. 3 of a call: one set per device for the whole process,
// made on first use and kept until the process ends. All handles share them, so
// that a process holds the caller's stream plus three - HIP gives it four hardware
// queues, and streams that share a queue run their kernels one after the other.
// Plain streams (default priority) that do not synchronise with stream 0. The order
// of a call's work is given by its own fork / join events, so calls on different
// handles may share the streams.
hipError_t bucket_stream(int device, int q, hipStream_t* out)
{
    static std::mutex mu;
    static std::vector<hipStream_t> pool;  // [device * kMax + q]
    std::lock_guard<std::mutex> lock(mu);
    const size_t at = (size_t)device * Buckets::kMax + (size_t)q;
    if (pool.size() <= at) pool.resize(at + 1, nullptr);
    if (!pool[at]) {
        const hipError_t e = hipStreamCreateWithFlags(&pool[at], hipStreamNonBlocking);
        if (e != hipSuccess) {
            pool[at] = nullptr;
            return e;
        }
    }
    *out = pool[at];
    return hipSuccess;
}

// Argument checks shared by the forward-backward entry points (B == 0 is valid:
// the caller then returns at once).
lfmmi_status check_call(const lfmmi_graph* h, const float* logits, const int32_t* lengths,
                        int32_t B, int32_t T, int32_t P, float leak, float grad_scale,
                        const float* objf, const float* grad)
{
    if (!h) return fail(LFMMI_ERR_INVALID_ARG, "graph is null");
    if (!h->uploaded) return fail(LFMMI_ERR_INVALID_ARG, "graph was packed but not uploaded");
    if (B < 0 || T < 0) return fail(LFMMI_ERR_INVALID_ARG, "B and T must be >= 0");
    if (P != h->num_pdfs) return fail(LFMMI_ERR_INVALID_ARG, "P differs from the graph's num_pdfs");
    if (!(leak >= 0.f) || !(leak < INFINITY)) return fail(LFMMI_ERR_INVALID_ARG, "leak must be finite and >= 0");
    if (!(grad_scale == grad_scale)) return fail(LFMMI_ERR_INVALID_ARG, "grad_scale is NaN");
    if (h->num_graphs != 1 && h->num_graphs != B)
        return fail(LFMMI_ERR_INVALID_ARG, "a batch handle needs one graph per sequence");
    if (B == 0) return LFMMI_OK;
    if (!lengths || !objf) return fail(LFMMI_ERR_INVALID_ARG, "lengths / objf is null");
    if (T > 0 && (!logits || !grad)) return fail(LFMMI_ERR_INVALID_ARG, "logits / grad is null");
    if (B > 32767) return fail(LFMMI_ERR_UNSUPPORTED, "B exceeds 32767");
    for (int32_t b = 0; b < B; ++b)
        if (lengths[b] < 0 || lengths[b] > T)
            return fail(LFMMI_ERR_INVALID_ARG, "lengths[" + std::to_string(b) + "] outside [0, T]");
    // the packed graph and the workspace live on the device of the upload
    int current = -1;
    const hipError_t e = hipGetDevice(&current);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (current != h->device)
        return fail(LFMMI_ERR_INVALID_ARG, "the graph was uploaded to device " +
                                               std::to_string(h->device) + ", the current device is " +
                                               std::to_string(current));
    return LFMMI_OK;
}

// Where the parts of a call's workspace lie (byte offsets): the descriptors
// first (what a call stages from the host), then what the kernels produce.
struct CallLayout {
    size_t at_seqs, at_order, stage_need, at_emis, at_rowmax, at_alpha, at_beta, at_scal, at_cfac,
        at_zfin, at_status, total;
    int64_t scal_total;
};

// a_at / b_at: values in all alpha / beta trellises; s_at: frames + sequences.
CallLayout layout_call(const lfmmi_graph* h, int32_t B, int32_t T, int32_t P, int64_t a_at,
                       int64_t b_at, int64_t s_at)
{
    CallLayout l{};
    size_t total = 0;
    l.at_seqs = reserve<SeqDesc>(&total, B);
    l.at_order = reserve<int32_t>(&total, (size_t)2 * B);
    l.stage_need = total;
    l.at_emis = reserve<float>(&total, (size_t)B * T * P);
    l.at_rowmax = reserve<float>(&total, (size_t)B * T);
    const size_t real = h->wide ? 2 : 1;  // floats per value
    l.at_alpha = reserve<float>(&total, (size_t)a_at * real);
    l.at_beta = reserve<float>(&total, (size_t)b_at * real);
    l.at_scal = reserve<float>(&total, (size_t)4 * s_at * real);
    l.at_cfac = reserve<float>(&total, (size_t)s_at * real);
    l.at_zfin = reserve<float>(&total, (size_t)2 * B * real);
    l.at_status = reserve<int32_t>(&total, B);
    l.total = total;
    l.scal_total = s_at;
    return l;
}

void fill_params(lfmmi_graph* h, const CallLayout& lay, unsigned char* ws,
                 const float* logits, int32_t B, int32_t T, int32_t P, float leak,
                 float grad_scale, int accumulate, float* objf, float* grad, int32_t* status,
                 FbParams* out, LaunchShape* shape_out)
{
    FbParams& p = *out;
    p.g = h->dg;
    p.seqs = reinterpret_cast<const SeqDesc*>(ws + lay.at_seqs);
    p.order = reinterpret_cast<const int32_t*>(ws + lay.at_order);
    p.logits = logits;
    p.emis = reinterpret_cast<float*>(ws + lay.at_emis);
    p.rowmax = reinterpret_cast<float*>(ws + lay.at_rowmax);
    p.emis_ready = 0;
    if (h->borrow_emis) {  // the other pass of a full-loss call computed them (read only here)
        p.emis = const_cast<float*>(h->borrow_emis);
        p.rowmax = const_cast<float*>(h->borrow_rowmax);
        p.emis_ready = 1;
        h->last_emis = nullptr;
    } else {
        h->last_emis = p.emis;
        h->last_rowmax = p.rowmax;
        h->last_emis_count = (size_t)B * T * P;
    }
    p.alpha = ws + lay.at_alpha;
    p.beta = ws + lay.at_beta;
    p.scal = ws + lay.at_scal;
    p.cfac = ws + lay.at_cfac;
    p.zfin = ws + lay.at_zfin;
    p.wide = h->wide ? 1 : 0;
    p.done = reinterpret_cast<int32_t*>(ws + lay.at_status);
    p.status_out = status;
    p.objf = objf;
    p.grad = grad;
    p.scal_total = lay.scal_total;
    p.B = B;
    p.T = T;
    p.P = P;
    p.lds_rows = std::max(h->max_rows_f, h->max_rows_b);
    p.lds_rows_occ_a = h->max_rows_f;
    p.lds_rows_occ_b = h->max_rows_b;
    p.lds_rows_occ = h->max_rows_occ;
    p.accumulate = accumulate ? 1 : 0;
    p.leak = leak;
    p.grad_scale = grad_scale;

    LaunchShape& shape = *shape_out;
    shape.rec_threads = h->rec_waves * kLanes;
    shape.rec_nslot = h->rec_nslot;
    shape.rec_yrep = h->rec_yrep ? 1 : 0;
    shape.rec_hybrid = h->rec_hybrid;
    shape.rec_hubs = h->rec_hubs ? 1 : 0;
    shape.rec_grouped = h->rec_grouped ? 1 : 0;
    shape.profile_rec_only = h->profile == 2 ? 1 : 0;
    shape.rec_has_wb = h->has_wb ? 1 : 0;
    shape.occ_threads = h->occ_waves * kLanes;
    shape.occ_frames = std::max(1, env_int("LFMMI_OCC_FRAMES", 4));
    // the plane-layout occupancy kernel (several frames per arc record) when it fits
    {
        const int most = env_int("LFMMI_OCC_MULTI", 4);  // 0: the frame-at-a-time kernel
        shape.occ_multi = h->wide || most <= 0
                              ? 0
                              : occ_plane_frames(std::max(h->max_rows_f, h->max_rows_b),
                                                 h->max_rows_occ, most);
    }
    // groups of frames per workgroup: with one frame per group a workgroup takes four,
    // with two frames of large planes two, which spreads its start-up cost and lets it
    // fetch the next group's rows early (the variants with small planes do not: two of
    // their workgroups share a compute unit and cover each other's loads)
    const bool large_planes = std::max(h->max_rows_f, h->max_rows_b) * 4 > 16384;
    shape.occ_groups = std::max(
        1, env_int("LFMMI_OCC_GROUPS",
                   shape.occ_multi == 1 ? 4 : (shape.occ_multi == 2 && large_planes ? 2 : 1)));
}

}  // namespace

extern "C" {

const char* lfmmi_last_error(void) { return g_error.c_str(); }

lfmmi_status lfmmi_graph_pack_batch(int32_t n, int32_t num_pdfs, const int64_t* state_off,
                                    const int64_t* arc_off, const int32_t* src,
                                    const int32_t* dst, const int32_t* pdf, const float* logw,
                                    const float* init_prob, const float* final_prob,
                                    lfmmi_graph** out)
{
    return pack_all(n, num_pdfs, state_off, arc_off, src, dst, pdf, logw, init_prob,
                    final_prob, out);
}

lfmmi_status lfmmi_graph_pack(int32_t num_states, int32_t num_pdfs, int64_t num_arcs,
                              const int32_t* src, const int32_t* dst, const int32_t* pdf,
                              const float* logw, const float* init_prob,
                              const float* final_prob, lfmmi_graph** out)
{
    const int64_t so[2] = {0, num_states}, ao[2] = {0, num_arcs};
    if (num_arcs < 0) return fail(LFMMI_ERR_INVALID_ARG, "num_arcs must be >= 0");
    return pack_all(1, num_pdfs, so, ao, src, dst, pdf, logw, init_prob, final_prob, out);
}

lfmmi_status lfmmi_graph_upload(lfmmi_graph* graph)
{
    if (!graph) return fail(LFMMI_ERR_INVALID_ARG, "graph is null");
    return upload(graph);
}

lfmmi_status lfmmi_graph_create(int32_t num_states, int32_t num_pdfs, int64_t num_arcs,
                                const int32_t* src, const int32_t* dst, const int32_t* pdf,
                                const float* logw, const float* init_prob,
                                const float* final_prob, lfmmi_graph** out)
{
    lfmmi_status st = lfmmi_graph_pack(num_states, num_pdfs, num_arcs, src, dst, pdf, logw,
                                       init_prob, final_prob, out);
    if (st != LFMMI_OK) return st;
    st = upload(*out);
    if (st != LFMMI_OK) { lfmmi_graph_destroy(*out); *out = nullptr; }
    return st;
}

lfmmi_status lfmmi_graph_create_batch(int32_t n, int32_t num_pdfs, const int64_t* state_off,
                                      const int64_t* arc_off, const int32_t* src,
                                      const int32_t* dst, const int32_t* pdf,
                                      const float* logw, const float* init_prob,
                                      const float* final_prob, lfmmi_graph** out)
{
    lfmmi_status st = pack_all(n, num_pdfs, state_off, arc_off, src, dst, pdf, logw,
                               init_prob, final_prob, out);
    if (st != LFMMI_OK) return st;
    st = upload(*out);
    if (st != LFMMI_OK) { lfmmi_graph_destroy(*out); *out = nullptr; }
    return st;
}

void lfmmi_graph_destroy(lfmmi_graph* h)
{
    if (!h) return;
    if (h->uploaded || h->ws || h->stage) {
        (void)hipDeviceSynchronize();
        if (h->dev_base) (void)hipFree(h->dev_base);
        if (h->ws) (void)hipFree(h->ws);
        if (h->stage) (void)hipHostFree(h->stage);
        if (h->stage_done) (void)hipEventDestroy(h->stage_done);
        for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
        for (hipEvent_t e : h->ev_free) (void)hipEventDestroy(e);
        for (int q = 1; q < Buckets::kMax; ++q) {
            if (h->join[q]) (void)hipEventDestroy(h->join[q]);
        }
        if (h->fork) (void)hipEventDestroy(h->fork);
    }
    delete h;
}

lfmmi_status lfmmi_forward_backward(const lfmmi_graph* graph, const float* logits,
                                    const int32_t* lengths, int32_t B, int32_t T, int32_t P,
                                    float leak, float grad_scale, int accumulate, float* objf,
                                    float* grad, int32_t* status, void* hip_stream)
{
    lfmmi_graph* h = const_cast<lfmmi_graph*>(graph);  // the workspace is mutable state
    lfmmi_status st = check_call(h, logits, lengths, B, T, P, leak, grad_scale, objf, grad);
    if (st != LFMMI_OK || B == 0) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;

    // ---- per-sequence descriptors and the launch order (longest first)
    std::vector<SeqDesc> seqs(B);
    int64_t a_at = 0, b_at = 0, s_at = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t g = h->num_graphs == 1 ? 0 : b;
        const int64_t rf = h->packed[g].ord[0].num_slices * kLanes;
        const int64_t rb = h->packed[g].ord[1].num_slices * kLanes;
        seqs[b].alpha_at = a_at;
        seqs[b].beta_at = b_at;
        seqs[b].T = lengths[b];
        seqs[b].graph = g;
        seqs[b].scal_at = (int32_t)s_at;
        seqs[b].pad = 0;
        a_at += rf * (lengths[b] + 1);
        b_at += rb * (lengths[b] + 1);
        s_at += lengths[b] + 1;
    }
    if (s_at > (int64_t)1 << 30) return fail(LFMMI_ERR_UNSUPPORTED, "too many frames in one call");
    std::vector<int32_t> by_len(B);
    std::iota(by_len.begin(), by_len.end(), 0);
    std::stable_sort(by_len.begin(), by_len.end(), [&](int32_t x, int32_t y) {
        const int64_t wx = (int64_t)lengths[x] * h->packed[seqs[x].graph].num_arcs;
        const int64_t wy = (int64_t)lengths[y] * h->packed[seqs[y].graph].num_arcs;
        return wx != wy ? wx > wy : lengths[x] > lengths[y];
    });
    std::vector<int32_t> order((size_t)2 * B);
    for (int32_t i = 0; i < B; ++i) {
        order[(size_t)2 * i] = by_len[i] << 1;
        order[(size_t)2 * i + 1] = (by_len[i] << 1) | 1;
    }

    const CallLayout lay = layout_call(h, B, T, P, a_at, b_at, s_at);
    const size_t total = lay.total, stage_need = lay.stage_need;
    if (total > h->ws_bytes) {
        h->desc_lengths.clear();
        h->desc_T = -1;
        if (h->ws) {
            (void)hipDeviceSynchronize();
            (void)hipFree(h->ws);
            h->ws = nullptr;
            h->ws_bytes = 0;
        }
        // an eighth more than asked for: batches whose lengths vary a little from call to
        // call (the usual training loop) then settle after a few calls instead of
        // synchronising and reallocating at every new maximum
        size_t want = total + total / 8;
        if ((e = hipMalloc(&h->ws, want)) != hipSuccess) {
            want = total;
            e = hipMalloc(&h->ws, want);
        }
        if (e != hipSuccess) {
            h->ws = nullptr;
            return fail(LFMMI_ERR_OOM, "workspace of " + std::to_string(total) +
                                           " bytes: " + hipGetErrorString(e));
        }
        h->ws_bytes = want;
    }
    // descriptors depend on the lengths and T only: a call with the same ones as
    // the last finds them on the device already
    const bool same_desc = h->desc_T == T && (int32_t)h->desc_lengths.size() == B &&
                           std::equal(h->desc_lengths.begin(), h->desc_lengths.end(), lengths);
    unsigned char* ws = static_cast<unsigned char*>(h->ws);
    if (!same_desc) {
        if (stage_need > h->stage_bytes) {
            if (h->stage) {
                if (h->stage_pending) (void)hipEventSynchronize(h->stage_done);
                (void)hipHostFree(h->stage);
                h->stage = nullptr;
                h->stage_bytes = 0;
            }
            if ((e = hipHostMalloc(&h->stage, stage_need, hipHostMallocDefault)) != hipSuccess) {
                h->stage = nullptr;
                return fail(LFMMI_ERR_OOM, std::string("hipHostMalloc: ") + hipGetErrorString(e));
            }
            h->stage_bytes = stage_need;
        }
        if (!h->stage_done &&
            (e = hipEventCreateWithFlags(&h->stage_done, hipEventDisableTiming)) != hipSuccess)
            return fail_hip(e, "hipEventCreate");
        if (h->stage_pending) {
            // the previous call's descriptor copy must have left the staging buffer
            if ((e = hipEventSynchronize(h->stage_done)) != hipSuccess)
                return fail_hip(e, "hipEventSynchronize");
            h->stage_pending = false;
        }
        unsigned char* stg = static_cast<unsigned char*>(h->stage);
        std::memcpy(stg + lay.at_seqs, seqs.data(), sizeof(SeqDesc) * B);
        std::memcpy(stg + lay.at_order, order.data(), sizeof(int32_t) * 2 * B);
        h->desc_lengths.clear();
        h->desc_T = -1;
        if ((e = hipMemcpyAsync(ws, stg, stage_need, hipMemcpyHostToDevice, stream)) != hipSuccess)
            return fail_hip(e, "hipMemcpyAsync");
        if ((e = hipEventRecord(h->stage_done, stream)) != hipSuccess)
            return fail_hip(e, "hipEventRecord");
        h->stage_pending = true;
        h->desc_lengths.assign(lengths, lengths + B);
        h->desc_T = T;
    }

    FbParams p{};
    LaunchShape shape;
    fill_params(h, lay, ws, logits, B, T, P, leak, grad_scale, accumulate, objf, grad, status, &p,
                &shape);

    // ---- buckets of sequences that run concurrently (longest sequences first):
    // an eighth, a quarter, a quarter and the rest, so that the bucket that ends
    // last has little occupancy work left to do on its own
    Buckets bk;
    {
        int want = std::min(env_int("LFMMI_BUCKETS", Buckets::kMax), (int)Buckets::kMax);
        want = std::max(1, std::min(want, B / 2));
        if (T == 0) want = 1;
        static const double upto[Buckets::kMax][Buckets::kMax] = {
            {1.0, 1.0, 1.0, 1.0}, {0.25, 1.0, 1.0, 1.0}, {0.15, 0.5, 1.0, 1.0}, {0.125, 0.375, 0.625, 1.0}};
        double fr[Buckets::kMax];
        for (int q = 0; q < Buckets::kMax; ++q) fr[q] = upto[want - 1][q];
        if (const char* txt = std::getenv("LFMMI_BUCKET_FRACS")) {  // "f0,f1,f2": tuning
            const char* c = txt;
            for (int q = 0; q + 1 < want && *c; ++q) {
                char* stop = nullptr;
                const double v = std::strtod(c, &stop);
                if (stop == c) break;
                if (v > 0.0 && v <= 1.0) fr[q] = v;
                c = *stop == ',' ? stop + 1 : stop;
            }
        }
        bk.n = want;
        int at = 0;
        for (int q = 0; q < want; ++q) {
            int end = q == want - 1 ? B : (int)std::lround(fr[q] * B);
            end = std::max(at + 1, std::min(end, B - (want - 1 - q)));
            bk.first[q] = at;
            bk.count[q] = end - at;
            for (int i = at; i < end; ++i) bk.tmax[q] = std::max(bk.tmax[q], lengths[by_len[i]]);
            at = end;
        }
        if (want > 1) {
            if (!h->fork &&
                (e = hipEventCreateWithFlags(&h->fork, hipEventDisableTiming)) != hipSuccess)
                return fail_hip(e, "hipEventCreate");
            for (int q = 1; q < want; ++q) {
                // plain streams (default priority) that do not synchronise with stream 0
                hipStream_t aux = nullptr;
                if ((e = bucket_stream(h->device, q, &aux)) != hipSuccess)
                    return fail_hip(e, "hipStreamCreate");
                if (!h->join[q] &&
                    (e = hipEventCreateWithFlags(&h->join[q], hipEventDisableTiming)) != hipSuccess)
                    return fail_hip(e, "hipEventCreate");
                bk.streams[q] = aux;
                bk.join[q] = h->join[q];
            }
            bk.fork = h->fork;
        }
    }

    hipEvent_t* ev = nullptr;
    if (h->profile) {
        const size_t first = h->ev.size(), count = 4 * (size_t)bk.n;
        h->ev.resize(first + count, nullptr);
        for (size_t i = first; i < first + count; ++i)
            if (!h->ev_free.empty()) {
                h->ev[i] = h->ev_free.back();
                h->ev_free.pop_back();
            } else if ((e = hipEventCreate(&h->ev[i])) != hipSuccess) {
                for (size_t j = first; j < i; ++j) (void)hipEventDestroy(h->ev[j]);
                h->ev.resize(first);
                return fail_hip(e, "hipEventCreate");
            }
        h->ev_buckets.push_back(bk.n);
        ev = h->ev.data() + first;
    }
    if ((e = launch_forward_backward(p, shape, stream, ev, bk)) != hipSuccess)
        return fail_hip(e, "kernel launch");
    return LFMMI_OK;
}

lfmmi_status lfmmi_forward_backward_static(const lfmmi_graph* graph, const float* logits,
                                           const int32_t* lengths, int32_t B, int32_t T,
                                           int32_t P, float leak, float grad_scale,
                                           int accumulate, float* objf, float* grad,
                                           int32_t* status, void* hip_stream)
{
    lfmmi_graph* h = const_cast<lfmmi_graph*>(graph);
    lfmmi_status st = check_call(h, logits, lengths, B, T, P, leak, grad_scale, objf, grad);
    if (st != LFMMI_OK || B == 0) return st;
    if (B > LFMMI_STATIC_MAX_BATCH)
        return fail(LFMMI_ERR_UNSUPPORTED, "B = " + std::to_string(B) + " exceeds the " +
                                               std::to_string(LFMMI_STATIC_MAX_BATCH) +
                                               " sequences of the allocation-free entry point");
    int64_t a_at = 0, b_at = 0, s_at = 0;
    int32_t t_most = 0;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t g = h->num_graphs == 1 ? 0 : b;
        a_at += (int64_t)h->packed[g].ord[0].num_slices * kLanes * (lengths[b] + 1);
        b_at += (int64_t)h->packed[g].ord[1].num_slices * kLanes * (lengths[b] + 1);
        s_at += lengths[b] + 1;
        t_most = std::max(t_most, lengths[b]);
    }
    const CallLayout lay = layout_call(h, B, T, P, a_at, b_at, s_at);
    if (lay.total > (size_t)LFMMI_STATIC_WORKSPACE_BYTES)
        return fail(LFMMI_ERR_UNSUPPORTED,
                    "this call needs " + std::to_string(lay.total) + " bytes of workspace, the "
                    "allocation-free entry point holds " +
                    std::to_string((size_t)LFMMI_STATIC_WORKSPACE_BYTES));
    // the device's copy of the static array, looked up when the graph was uploaded
    unsigned char* ws = static_cast<unsigned char*>(static_workspace(h->device));
    if (!ws) return fail(LFMMI_ERR_HIP, "the static workspace of this device was not found");

    FbParams p{};
    LaunchShape shape;
    fill_params(h, lay, ws, logits, B, T, P, leak, grad_scale, accumulate, objf, grad, status, &p,
                &shape);
    shape.profile_rec_only = 0;
    Buckets bk;  // one bucket, on the caller's stream: no stream or event of the library's
    bk.n = 1;
    bk.first[0] = 0;
    bk.count[0] = B;
    bk.tmax[0] = t_most;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    // descriptors and launch order are written on the device, from the lengths
    // passed as a kernel argument (no host-to-device copy to stage)
    if ((e = launch_describe(p, lengths, h->num_graphs, stream)) != hipSuccess)
        return fail_hip(e, "kernel launch");
    if ((e = launch_forward_backward(p, shape, stream, nullptr, bk)) != hipSuccess)
        return fail_hip(e, "kernel launch");
    return LFMMI_OK;
}

lfmmi_status lfmmi_loss(const lfmmi_graph* num, const lfmmi_graph* den, const float* logits,
                        const int32_t* lengths, int32_t B, int32_t T, int32_t P, float leak,
                        float* objf, float* grad, int32_t* status, void* hip_stream)
{
    if (!num || !den) return fail(LFMMI_ERR_INVALID_ARG, "graph is null");
    if (num == den) return fail(LFMMI_ERR_INVALID_ARG, "numerator and denominator share a handle");
    // Numerators (+1, overwrite), then the denominator (-1, accumulate), one after the
    // other on the caller's stream. Running the two passes on streams of their own
    // was measured slower (see the header): without stream priorities the numerators'
    // workgroups take compute units from the denominator's longest sequences, whose
    // recursion is the critical path of the call.
    lfmmi_graph* hn = const_cast<lfmmi_graph*>(num);
    lfmmi_graph* hd = const_cast<lfmmi_graph*>(den);
    hn->last_emis = nullptr;
    lfmmi_status st = lfmmi_forward_backward(num, logits, lengths, B, T, P, leak, 1.f, 0, objf,
                                             grad, status, hip_stream);
    if (st != LFMMI_OK) return st;
    // exp(logit - row maximum) and the row maxima are the same for both passes: the
    // denominator's reads what the numerators' pass left in its workspace (same
    // stream, so it is complete; same B, T, P, so the layout is the same)
    if (hn->last_emis && hn->last_emis_count == (size_t)B * T * P &&
        env_int("LFMMI_SHARE_EMIS", 1) != 0) {
        hd->borrow_emis = hn->last_emis;
        hd->borrow_rowmax = hn->last_rowmax;
    }
    st = lfmmi_forward_backward(den, logits, lengths, B, T, P, leak, -1.f, 1, objf, grad, status,
                                hip_stream);
    hd->borrow_emis = nullptr;
    hd->borrow_rowmax = nullptr;
    return st;
}

lfmmi_status lfmmi_graph_info(const lfmmi_graph* h, int64_t info[8])
{
    if (!h || !info) return fail(LFMMI_ERR_INVALID_ARG, "null argument");
    info[0] = h->num_graphs;
    info[1] = h->num_pdfs;
    info[2] = h->total_states;
    info[3] = h->total_arcs;
    info[4] = h->rec_waves;
    info[5] = h->occ_waves;
    info[6] = (h->uploaded ? 1 : 0) | (h->wide ? 2 : 0) | (h->rec_grouped ? 4 : 0);
    info[7] = (int64_t)h->ws_bytes;
    return LFMMI_OK;
}

lfmmi_status lfmmi_graph_ordering_info(const lfmmi_graph* h, int32_t g, int32_t ord,
                                       int64_t info[12])
{
    if (!h || !info) return fail(LFMMI_ERR_INVALID_ARG, "null argument");
    if (g < 0 || g >= h->num_graphs || ord < 0 || ord > 2)
        return fail(LFMMI_ERR_INVALID_ARG, "graph or ordering index out of range");
    const Ordering& o = h->packed[g].ord[ord];
    info[0] = o.num_rows;
    info[1] = o.num_slices;
    info[2] = o.num_waves;
    info[3] = o.total_slots;
    info[4] = o.max_wave_slots;
    info[5] = ord < 2 ? h->rec_nslot : 0;
    info[6] = ord < 2 && h->rec_yrep ? 1 : 0;
    info[7] = o.has_wb;
    info[8] = o.gather_cycles;
    info[9] = ord < 2 ? o.closing_slots : 0;
    info[10] = 0;
    for (int32_t f : o.slice_hub) info[10] += f != 0;
    // rows one state vector of the chosen recursion kernel's fixed LDS map holds
    info[11] = ord == 2 || h->rec_nslot == 0 ? 0
               : h->rec_hybrid == 2          ? 12288
                                             : (h->wide ? 4096 : 8192);
    return LFMMI_OK;
}

lfmmi_status lfmmi_graph_ordering_copy(const lfmmi_graph* h, int32_t g, int32_t ord,
                                       int32_t* slice_off, int32_t* wave_first, uint32_t* key,
                                       float* w, int32_t* row_id, int32_t* slice_hub)
{
    if (!h) return fail(LFMMI_ERR_INVALID_ARG, "null argument");
    if (g < 0 || g >= h->num_graphs || ord < 0 || ord > 2)
        return fail(LFMMI_ERR_INVALID_ARG, "graph or ordering index out of range");
    const Ordering& o = h->packed[g].ord[ord];
    if (slice_off) std::memcpy(slice_off, o.slice_off.data(), o.slice_off.size() * 4);
    if (wave_first) std::memcpy(wave_first, o.wave_first.data(), o.wave_first.size() * 4);
    if (key) std::memcpy(key, o.key.data(), o.key.size() * 4);
    if (w) std::memcpy(w, o.w.data(), o.w.size() * 4);
    if (row_id) std::memcpy(row_id, o.row_id.data(), o.row_id.size() * 4);
    if (slice_hub)
        for (int32_t sl = 0; sl < o.num_slices; ++sl)
            slice_hub[sl] = (size_t)sl < o.slice_hub.size() ? o.slice_hub[sl] : 0;
    return LFMMI_OK;
}

lfmmi_status lfmmi_profile_enable(lfmmi_graph* h, int enable)
{
    if (!h) return fail(LFMMI_ERR_INVALID_ARG, "graph is null");
    if (enable < 0 || enable > 2) return fail(LFMMI_ERR_INVALID_ARG, "enable must be 0, 1 or 2");
    if (enable != h->profile && !h->ev_buckets.empty())
        return fail(LFMMI_ERR_INVALID_ARG, "read the recorded calls before changing the level");
    h->profile = enable;
    return LFMMI_OK;
}

lfmmi_status lfmmi_profile_read(lfmmi_graph* h, float ms[4], int32_t* calls, int32_t* launches)
{
    if (!h || !ms) return fail(LFMMI_ERR_INVALID_ARG, "null argument");
    const size_t n = h->ev_buckets.size();
    if (calls) *calls = (int32_t)n;
    if (launches) *launches = 0;
    for (int i = 0; i < 4; ++i) ms[i] = 0.f;
    if (n == 0) return fail(LFMMI_ERR_INVALID_ARG, "no profiled call to read");
    lfmmi_status st = LFMMI_OK;
    hipError_t e;
    double sum[4] = {0, 0, 0, 0};
    int64_t runs = 0;
    auto elapsed = [&](size_t from, size_t to, double* acc) {
        float t = 0.f;
        if ((e = hipEventSynchronize(h->ev[to])) != hipSuccess ||
            (e = hipEventElapsedTime(&t, h->ev[from], h->ev[to])) != hipSuccess) {
            st = fail_hip(e, "hipEventElapsedTime");
            return;
        }
        *acc += t;
    };
    size_t at = 0;
    for (size_t c = 0; c < n && st == LFMMI_OK; ++c) {
        for (int q = 0; q < h->ev_buckets[c] && st == LFMMI_OK; ++q) {
            const size_t b0 = at + 4 * (size_t)q;
            if (h->profile != 2) elapsed(b0, b0 + 1, &sum[0]);
            elapsed(b0 + 1, b0 + 2, &sum[1]);
            if (h->profile != 2) elapsed(b0 + 2, b0 + 3, &sum[3]);
            ++runs;
        }
        at += 4 * (size_t)h->ev_buckets[c];
    }
    h->ev_free.insert(h->ev_free.end(), h->ev.begin(), h->ev.end());  // kept for the next calls
    h->ev.clear();
    h->ev_buckets.clear();
    if (st == LFMMI_OK) {
        for (int i = 0; i < 4; ++i) ms[i] = (float)(sum[i] / (double)runs);
        if (launches) *launches = (int32_t)runs;
    }
    return st;
}

}  // extern "C"
