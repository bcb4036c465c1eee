/*
 * lfmmi.h - C ABI of the MI355X (gfx950) LF-MMI forward-backward library.
 *
 * The library computes, for a batch of unequal-length sequences, the HMM
 * forward-backward over a graph shared by the batch (denominator) or over one
 * graph per sequence (numerators): the per-sequence log-likelihood
 * log P(X | G) of Eq. 2 and the pdf occupancies gamma of Eq. 3, which are the
 * derivative of that log-likelihood with respect to the network output.
 *
 * Model (Section 3.3, Section 3.4 / Algorithm 1):
 *   an arc goes from state src to state dst, emits pdf-id pdf and has
 *   probability w = exp(logw); frame t of a sequence multiplies an arc by
 *   exp(logits[b, t, pdf]); a graph has initial probabilities init_prob[s]
 *   (a unique initial state is the one-hot case) and final probabilities
 *   final_prob[s], applied at the sequence's own last frame. The leaky HMM the
 *   paper refers to is taken as: at t = 0 and after every frame each state s
 *   additionally receives leak * (total mass) * init_prob[s].
 *
 * Conventions: every function returns an lfmmi_status (never throws, never
 * aborts); on failure lfmmi_last_error() describes the reason (thread-local).
 * Inputs are never modified. "HOST" / "DEVICE" says where a pointer lives.
 */
#ifndef LFMMI_H
#define LFMMI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lfmmi_graph lfmmi_graph; /* opaque; owns host and device copies */

typedef enum {
    LFMMI_OK = 0,
    LFMMI_ERR_INVALID_ARG = 1, /* null pointer, negative size, shape mismatch   */
    LFMMI_ERR_BAD_GRAPH = 2,   /* state / pdf id out of range, non-finite weight */
    LFMMI_ERR_OOM = 3,         /* host or device allocation failed               */
    LFMMI_ERR_HIP = 4,         /* a HIP runtime call failed (no GPU, launch...)  */
    LFMMI_ERR_UNSUPPORTED = 5  /* size beyond what the kernels hold in LDS       */
} lfmmi_status;

/*
 * Graph packing (Section 3.3: the transition list sorted by from-state and by
 * to-state with per-state index ranges; here three sliced-ELL orderings -
 * by to-state, by from-state, by pdf-id - built once on the host).
 *
 * All pointers HOST, copied. Arcs in any order, duplicates allowed.
 *   src, dst [num_arcs] in [0, num_states); pdf [num_arcs] in [0, num_pdfs);
 *   logw [num_arcs] natural-log weight, finite (drop an arc instead of -inf);
 *   init_prob, final_prob [num_states] linear, >= 0, finite, not normalised.
 * Limits (the recursion keeps two state vectors and two emission rows in the
 * 160 KB of LDS of a compute unit): num_states <= 16384, num_pdfs <= 16384 and
 * 8 * (num_states rounded up to 64) + 8 * (num_pdfs rounded up to 64) + 128
 * <= 163840 bytes, else LFMMI_ERR_UNSUPPORTED. num_arcs may be 0.
 * When some state has final_prob == 0 or init_prob == 0 (left-to-right graphs:
 * numerators, or any graph entered through one state) the state vectors, trellis
 * and scales are kept in fp64 and the limit above counts 16 bytes per state;
 * when every state is initial and final they are fp32. The environment variable
 * LFMMI_PRECISION=32 or 64, read when a graph is packed, overrides that choice:
 * it changes results (32 on a left-to-right graph can lose posterior mass to
 * underflow, which lfmmi_forward_backward then reports in status).
 * lfmmi_graph_create packs and uploads to the current HIP device.
 * lfmmi_graph_pack only packs (no HIP call): for host-side inspection; such a
 * handle is refused by lfmmi_forward_backward until lfmmi_graph_upload.
 */
lfmmi_status lfmmi_graph_create(int32_t num_states, int32_t num_pdfs, int64_t num_arcs,
                                const int32_t *src, const int32_t *dst,
                                const int32_t *pdf, const float *logw,
                                const float *init_prob, const float *final_prob,
                                lfmmi_graph **out);
lfmmi_status lfmmi_graph_pack(int32_t num_states, int32_t num_pdfs, int64_t num_arcs,
                              const int32_t *src, const int32_t *dst,
                              const int32_t *pdf, const float *logw,
                              const float *init_prob, const float *final_prob,
                              lfmmi_graph **out);

/*
 * n graphs in one handle (Section 3.3, the batch of numerator graphs; ragged
 * offsets instead of zero padding). Graph g owns states
 * [state_off[g], state_off[g+1]) of init_prob / final_prob and arcs
 * [arc_off[g], arc_off[g+1]); src / dst are local to the graph
 * (0 .. its state count - 1). All graphs share num_pdfs.
 */
lfmmi_status lfmmi_graph_create_batch(int32_t n, int32_t num_pdfs,
                                      const int64_t *state_off, const int64_t *arc_off,
                                      const int32_t *src, const int32_t *dst,
                                      const int32_t *pdf, const float *logw,
                                      const float *init_prob, const float *final_prob,
                                      lfmmi_graph **out);
lfmmi_status lfmmi_graph_pack_batch(int32_t n, int32_t num_pdfs,
                                    const int64_t *state_off, const int64_t *arc_off,
                                    const int32_t *src, const int32_t *dst,
                                    const int32_t *pdf, const float *logw,
                                    const float *init_prob, const float *final_prob,
                                    lfmmi_graph **out);
lfmmi_status lfmmi_graph_upload(lfmmi_graph *graph);
/* Frees host and device memory, including the cached workspace. NULL is a no-op.
 * Synchronises the device. */
void lfmmi_graph_destroy(lfmmi_graph *graph);

/*
 * Batched forward-backward (Algorithm 1 and its mirrored backward pass; Eq. 3).
 *
 *   graph    one graph (shared by all sequences) or a batch handle with n == B
 *            (graph b goes with sequence b).
 *   logits   DEVICE, float32 [B, T, P] row-major contiguous; rows t >= lengths[b]
 *            are never read.
 *   lengths  HOST, int32 [B], 0 <= lengths[b] <= T, any order.
 *   P        must equal the graph's num_pdfs.
 *   leak     leaky-HMM coefficient >= 0 (0 = plain HMM).
 *   objf     DEVICE float32 [B]:      objf[b]      (=|+=) grad_scale * log Z_b
 *   grad     DEVICE float32 [B, T, P]: grad[b,t,:] (=|+=) grad_scale * gamma_t
 *            accumulate == 0 overwrites (rows t >= lengths[b] become 0),
 *            accumulate != 0 adds (those rows are left alone). The full
 *            objective of Eq. 2 / Eq. 3 is: numerators with (+1, 0), then the
 *            denominator with (-1, 1).
 *   status   DEVICE int32 [B] or NULL: 0 ok; bit 0: zero total probability
 *            (log Z = -inf, gamma rows 0); bit 1: a non-finite logit was read
 *            (objf NaN, gamma rows 0); bit 2: the alpha pass and the beta pass
 *            disagree on log Z by more than 1e-3, i.e. one of them lost mass to
 *            underflow (fp32 state vectors with leak == 0, or forced by
 *            LFMMI_PRECISION=32): objf and gamma are written but not to be trusted.
 *   hip_stream  hipStream_t (NULL = default stream). The call only enqueues
 *            work; it does not synchronise. It may allocate (and so
 *            synchronise) when the handle's cached workspace has to grow.
 *            Internally the sequences are cut by length into up to four buckets
 *            whose kernels run on three streams the library keeps per device (default
 *            priority) between an event recorded on hip_stream and events
 *            hip_stream then waits for: all of the call's work is ordered on
 *            hip_stream as if it ran there. (The buckets overlap only while their
 *            streams sit on hardware queues of their own; HIP gives a process four
 *            by default, GPU_MAX_HW_QUEUES, and streams that share one run their
 *            kernels one after the other. LFMMI_BUCKETS=1..4 sets the bucket count.)
 *            A call with the same B, T and lengths as the handle's last one, and
 *            a workspace that is large enough already, copies nothing from the
 *            host and allocates nothing: it enqueues kernels, event records and
 *            event waits only, and may be captured into a HIP graph (relaxed
 *            capture mode, because of the library's own streams).
 * B == 0 or T == 0 with all lengths 0 are valid. Calls on one handle must be
 * ordered on one stream (they share the handle's workspace). The device the
 * graph was uploaded to must be the current one (LFMMI_ERR_INVALID_ARG if not).
 */
lfmmi_status lfmmi_forward_backward(const lfmmi_graph *graph, const float *logits,
                                    const int32_t *lengths, int32_t B, int32_t T,
                                    int32_t P, float leak, float grad_scale,
                                    int accumulate, float *objf, float *grad,
                                    int32_t *status, void *hip_stream);

/*
 * lfmmi_forward_backward for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments,
 * same results; the call's workspace (emission values, both trellises, per-frame
 * scales, descriptors) lies in a static device array of
 * LFMMI_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds from the
 * first graph upload on that GPU until the process ends, instead of in memory the
 * handle allocates. The call makes no hipMalloc / hipFree / hipHostMalloc, creates
 * no stream or event and copies nothing from the host: the lengths travel as a
 * kernel argument, all kernels run on hip_stream in one bucket, and there is no
 * per-kernel timing (lfmmi_profile_enable does not apply).
 * Limits: B <= LFMMI_STATIC_MAX_BATCH, and the workspace the call needs - about
 *   4 * B * T * P + 4 * sum_b (lengths[b] + 1) * (rows_fwd + rows_bwd + 5) bytes
 * (8 instead of 4 in the second term for fp64 graphs; rows = the padded row counts
 * lfmmi_graph_ordering_info reports as 64 * info[1]) - must fit the array, else
 * LFMMI_ERR_UNSUPPORTED with the two sizes in lfmmi_last_error().
 * All calls on one GPU share that GPU's array, whatever their handle or stream:
 * calls that overlap on one GPU race, so order them (one stream, or events).
 * Nothing in the array has to survive between calls; what must start at zero is
 * cleared by the call's own kernels.
 */
#define LFMMI_STATIC_WORKSPACE_BYTES (64u << 20)
#define LFMMI_STATIC_MAX_BATCH 256
lfmmi_status lfmmi_forward_backward_static(const lfmmi_graph *graph, const float *logits,
                                           const int32_t *lengths, int32_t B, int32_t T,
                                           int32_t P, float leak, float grad_scale,
                                           int accumulate, float *objf, float *grad,
                                           int32_t *status, void *hip_stream);

/*
 * The whole objective of Eq. 2 and its gradient, Eq. 3, in one call:
 *   objf[b]     = log P(X_b | numerator graph b) - log P(X_b | denominator graph)
 *   grad[b,t,:] = numerator occupancies - denominator occupancies (rows t >= lengths[b]: 0)
 *   status[b]   = the two passes' flags or-ed together (may be NULL)
 * exactly what lfmmi_forward_backward(num, ..., +1, 0, ...) followed by
 * lfmmi_forward_backward(den, ..., -1, 1, ...) leaves in the three arrays (bit for
 * bit), and enqueued the same way: the numerators' pass, then the denominator's,
 * on hip_stream. The emission values exp(logit - row maximum) are computed once,
 * by the numerators' pass; the denominator's reads them from that handle's
 * workspace. If the denominator's pass is refused (an error code comes back) the
 * numerators' pass is already enqueued and the three arrays are left holding its
 * results alone: treat them as undefined.
 * (Running the two passes beside each other on streams of their own
 * was built and measured 13 to 24 % slower on the 128-sequence workload: the
 * numerators' workgroups then take compute units from the denominator's longest
 * sequences, whose recursion decides when the call ends, and HIP streams of one
 * priority give no say in that.) num: a batch handle with B graphs (or one graph
 * for all); den: usually one shared graph; the two must be different handles.
 * Arguments and errors otherwise as lfmmi_forward_backward.
 */
lfmmi_status lfmmi_loss(const lfmmi_graph *num, const lfmmi_graph *den, const float *logits,
                        const int32_t *lengths, int32_t B, int32_t T, int32_t P, float leak,
                        float *objf, float *grad, int32_t *status, void *hip_stream);

/* Thread-local description of the last failure on this thread ("" if none). */
const char *lfmmi_last_error(void);

/* ---- introspection (host side; used by tests and the benchmark) ---------- */

enum { LFMMI_ORD_FWD = 0, LFMMI_ORD_BWD = 1, LFMMI_ORD_OCC = 2 };

/* info[0] number of graphs, [1] num_pdfs, [2] total states, [3] total arcs,
 * [4] waves per workgroup of the recursion kernel, [5] waves of the occupancy
 * kernel, [6] flags (bit 0: uploaded; bit 1: state vectors kept in fp64, which
 * is chosen when some state has final_prob 0 or init_prob 0; bit 2: every arc
 * carries the pdf-id of the state it enters - graphs expanded from HMMs whose
 * states emit, Section 4.2 - and the recursion runs without an emission gather per
 * arc: alpha multiplies a row by its emission once, beta folds the emission into
 * the stored vector), [7] workspace bytes held. */
lfmmi_status lfmmi_graph_info(const lfmmi_graph *graph, int64_t info[8]);

/* Packed ordering `ord` of graph `g`: info[0] rows, [1] slices (64 rows each),
 * [2] waves, [3] total slots (sum of slice widths), [4] max slots of one wave,
 * [5] arc slots the recursion kernel keeps in registers (0: streamed),
 * [6] 1 if the emission row is replicated per LDS bank, [7] 1 if the arcs carry
 * a per-arc leak factor (non-uniform init_prob), [8] modelled LDS cycles of the
 * gathers of one frame (per slot and half-wave, the largest number of distinct
 * addresses in one of the 32 banks), [9] 1 if every FWD / BWD slice ends in a
 * closing slot (packed so when init_prob is not uniform), [10] number of hub
 * slices (see below), [11] FWD / BWD: rows (slices * 64) one state vector of the
 * chosen recursion kernel's fixed LDS map holds, 0 when that kernel sizes its LDS
 * by the graph (arcs streamed). The kernel is chosen so that info[1] * 64 fits. */
lfmmi_status lfmmi_graph_ordering_info(const lfmmi_graph *graph, int32_t g,
                                       int32_t ord, int64_t info[12]);
/* Copies the packed ordering out (any pointer may be NULL):
 *   slice_off  [slices + 1] first slot of each slice
 *   wave_first [waves + 1]  first slice of each wave
 *   key, w     [total slots * 64] arc records, lane-minor; key = x-index * 4 in
 *              the low 16 bits, y-index * 4 in the high 16 bits; padding has w 0 (its
 *              key points wherever no bank conflict arises).
 *              With closing slots (info[9]) the last slot of every FWD / BWD
 *              slice holds no arc: its key is 0 and its w is the row's leak-dot
 *              weight (FWD: 1 on real rows; BWD: init_prob of the row's state)
 *   row_id     [slices * 64] the state (FWD: to-state, BWD: from-state) or
 *              pdf-id (OCC) a row stands for, -1 for padding rows
 *   slice_hub  [slices] 1 for a hub slice (FWD / BWD): a state with at least 64
 *              arcs and far more than the others gets a slice of its own; its
 *              row is that of lane 0, the arcs in all 64 lanes of the slice are
 *              its arcs (the kernels add the lanes' sums up), and the other 63
 *              rows are padding rows
 *   x-index / y-index: FWD (from-state in FWD numbering, pdf), BWD (to-state in
 *   BWD numbering, pdf), OCC (from-state in FWD numbering, to-state in BWD
 *   numbering), where a state's number in an ordering is the row it owns. */
lfmmi_status lfmmi_graph_ordering_copy(const lfmmi_graph *graph, int32_t g, int32_t ord,
                                       int32_t *slice_off, int32_t *wave_first,
                                       uint32_t *key, float *w, int32_t *row_id,
                                       int32_t *slice_hub);

/* Per-kernel timing with HIP events. While enabled, every lfmmi_forward_backward
 * on this handle records events around its kernels, on the streams they run on:
 * one emission, one recursion and one occupancy launch per bucket of sequences
 * (see lfmmi_forward_backward). enable: 0 off; 1 events around every kernel;
 * 2 around the recursion launches only (half the events: they cost about 3 % of
 * a call on the WSJ-shaped workload at level 1). Calls recorded at one level
 * must be read before the level changes. lfmmi_profile_read waits for the
 * events and returns mean durations per launch in milliseconds - ms[0] emission
 * (0 at level 2); [1] recursion (alpha and beta, and the scales, which the last
 * workgroup of a sequence computes); [2] 0; [3] occupancy + gradient (0 at
 * level 2) - with the number of calls in *calls and of launches of each kernel
 * in *launches (either may be NULL), then forgets them. Launches of one call
 * overlap: the means do not add up to the time of a call. */
lfmmi_status lfmmi_profile_enable(lfmmi_graph *graph, int enable);
lfmmi_status lfmmi_profile_read(lfmmi_graph *graph, float ms[4], int32_t *calls,
                                int32_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* LFMMI_H */
