// Plain-struct interface between the C ABI (api.cpp) and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace lfmmi {

// One packed ordering of one graph; offsets index the concatenated arrays of
// DeviceGraph.
struct OrdDesc {
    int32_t num_slices;     // rows = num_slices * 64
    int32_t num_waves;      // waves that own slices
    int32_t rec_at;         // first slot (units of 64 records) in recs
    int32_t slice_off_at;   // first entry in slice_off (num_slices + 1 entries)
    int32_t wave_first_at;  // first entry in wave_first (num_waves + 1 entries)
    int32_t vec_at;         // FWD/BWD: first row in vinit/va/vb/vfin; OCC: in row_slot
    int32_t max_wave_slots;
    int32_t total_slots;
    int32_t mask_at;        // FWD/BWD: first entry in wave_mask (num_waves entries)
    int32_t has_wb;         // FWD: the leak target differs per state
    float b_const;          // the leak target when it is one constant
    int32_t pdf_first_at;   // OCC: first entry in pdf_first (num_pdfs + 1 offsets, then the
                            // heavy-pdf list: count, row limit, pdf-ids)
    int32_t closing;        // FWD/BWD: slices end in a slot that holds the row's leak-dot weight
    float a_const;          // that weight when it is one constant (no closing slots)
};

struct DeviceGraph {
    const uint2* recs;          // {key, float bits of w}; slots 2q, 2q + 1 of lane l at
                                // [(q * 64 + l) * 2 + (0, 1)]
    const float* wb;            // w * b[from] per record (0 where unused), same indexing
    const uint64_t* wave_mask;  // closing-slot bit masks of the FWD/BWD waves
    const uint64_t* wave_hub;   // ... those of them that close a hub slice (same indexing)
    const int32_t* slice_hub;   // FWD/BWD: 1 for a hub slice; indexed like slice_off
    const int32_t* slice_off;   // slot offsets, local to the ordering
    const int32_t* wave_first;
    const float* vinit;
    const float* va;
    const float* vb;
    const float* vfin;
    const int32_t* row_pdf;     // FWD/BWD, graphs whose arcs take the pdf of the entered state:
                                // that pdf per row (indexed like vinit), else zeros
    const int32_t* pdf_first;   // OCC: the sums of pdf d's rows are words pdf_first[d] ..
                                // pdf_first[d + 1] - 1 of a frame's row sums
    const int32_t* row_slot;    // OCC: the word the sum of row (slice * 64 + lane) goes to
    const OrdDesc* ords;        // [num_graphs * 3]
};

struct SeqDesc {
    int64_t alpha_at;  // first float of this sequence's alpha trellis
    int64_t beta_at;
    int32_t T;         // frames of this sequence
    int32_t graph;     // graph index
    int32_t scal_at;   // first of its T + 1 per-frame scalars
    int32_t pad;
};

struct FbParams {
    DeviceGraph g;
    const SeqDesc* seqs;    // [B]
    const int32_t* order;   // [2B] (b << 1 | direction), longest sequences first
    int32_t seq_first;      // this launch covers order entries from 2 * seq_first on
    const float* logits;    // [B, T, P]
    float* emis;            // [B, T, P] exp(logit - row max)
    float* rowmax;          // [B, T]
    // the next five hold float, or double when `wide` is set
    void* alpha;            // ragged trellis, (T_b + 1) rows of rows_f values
    void* beta;
    void* scal;             // [4][scal_total] per frame: alpha n, alpha s, beta n, beta s
    void* cfac;             // [scal_total] occupancy scale of frame t at scal_at + t
    void* zfin;             // [2][B] closing dot products (alpha side, beta side)
    int32_t* done;          // [B] finished recursions of a sequence (0, 1, 2)
    int32_t* status_out;    // [B] or null
    float* objf;            // [B]
    float* grad;            // [B, T, P]
    int64_t scal_total;
    int32_t B, T, P;
    int32_t lds_rows;       // largest padded row count over the handle's graphs
    int32_t lds_rows_occ_a, lds_rows_occ_b;
    int32_t lds_rows_occ;   // largest padded OCC row count over the handle's graphs
    int32_t accumulate;
    int32_t wide;           // 1: state vectors, trellis and scales in fp64
    int32_t emis_ready;     // 1: emis / rowmax already hold this batch's values (the other
                            // pass of a full-loss call computed them): k_emit skips them
    float leak, grad_scale;
};

struct LaunchShape {
    int rec_threads;   // workgroup size of the recursion kernel
    int rec_nslot;     // arc slots held in registers per lane (0: streamed)
    int rec_yrep;      // emission row replicated across LDS banks
    int rec_has_wb;    // arcs carry a per-arc leak factor
    int rec_hubs;      // some graph of the handle has hub slices
    int profile_rec_only;  // of the four events per bucket record only those around k_rec
    int rec_hybrid;    // 1: only the first slots of a wave are register-resident;
                       // 2: the same, with the LDS map for up to 12288 states
    int rec_grouped = 0;  // arcs take the emission of the entered state: no emission gather
    int occ_threads;   // workgroup size of the occupancy kernel
    int occ_frames;    // frames per occupancy workgroup (frame-at-a-time kernel)
    int occ_multi;     // frames per record of the plane-layout occupancy kernel (0: not used)
    int occ_groups;    // groups of occ_multi frames per workgroup
};

// Sequences in launch order are cut into `n` consecutive buckets (longest
// first). Bucket 0 runs on the caller's stream, the others on streams[1..n-1]
// after the emission kernel, and the caller's stream waits for them at the end:
// short sequences finish the recursion early and their occupancy pass then
// overlaps the recursion of the long ones, which leaves compute units idle.
struct Buckets {
    static constexpr int kMax = 4;
    int n = 1;
    int first[kMax] = {0, 0, 0, 0};  // first sequence (index into the launch order)
    int count[kMax] = {0, 0, 0, 0};
    int tmax[kMax] = {0, 0, 0, 0};   // longest sequence of the bucket
    hipStream_t streams[kMax] = {nullptr, nullptr, nullptr, nullptr};  // [0] unused
    hipEvent_t fork = nullptr;                                        // n > 1 only
    hipEvent_t join[kMax] = {nullptr, nullptr, nullptr, nullptr};      // [0] unused
};

// Returns the first HIP error met (hipSuccess otherwise). ev, if non-null, holds
// 4 * n events: per bucket before, between and after its three kernels.
hipError_t launch_forward_backward(const FbParams& p, const LaunchShape& shape,
                                   hipStream_t stream, hipEvent_t* ev, const Buckets& bk);
hipError_t configure_kernels();

// The static device workspace of the allocation-free entry point: a file-scope
// device array of kStaticWorkspaceBytes, of which every GPU holds its own copy.
// find_static_workspace looks up the address of `device`'s copy (that device must
// be current); static_workspace returns it afterwards (null before).
constexpr size_t kStaticWorkspaceBytes = (size_t)64 << 20;
constexpr int kStaticMaxBatch = 256;
hipError_t find_static_workspace(int device);
void* static_workspace(int device);
// Writes the per-sequence descriptors and the launch order of a call (p.seqs,
// p.order, both inside the workspace) on the device, from the host array
// lengths[p.B] passed by value; p.B <= kStaticMaxBatch.
hipError_t launch_describe(const FbParams& p, const int32_t* lengths, int num_graphs,
                           hipStream_t stream);
// Dynamic LDS the recursion / occupancy kernels need.
size_t rec_lds_bytes(int lds_rows, int P, bool wide, bool yrep);
// Register-resident slot count the recursion kernel offers for this shape (0: none).
int rec_register_slots(bool wide, bool has_wb, bool yrep, bool hubs, int max_wave_slots,
                       int threads);
// Slots of the hybrid variant (a wave's leading slices in registers, the others
// streamed) for this kind of graph, 0 if there is none.
int rec_hybrid_slots(bool wide, bool has_wb, bool yrep, bool hubs, int map /* 1: 32 KB, 2: 48 KB */);
// Slots of the variant for graphs whose arcs take the pdf of the entered state
// (0: none for this shape), and the rows it stages emissions for with this many threads.
int rec_grouped_slots(bool wide, bool has_wb, int max_wave_slots, int threads);
int rec_grouped_max_rows(int threads);
size_t occ_lds_bytes(int rows_a, int rows_b, int occ_rows, bool wide);
int occ_plane_frames(int rows, int occ_rows, int most);
size_t occ_plane_lds_bytes(int rows, int occ_rows, int frames);

}  // namespace lfmmi
