// HIP kernels (gfx950) of the batched LF-MMI forward-backward.
//
// Pipeline of one call, per bucket of sequences (buckets run concurrently):
//   k_emit  e_t[d] = exp(x_t[d] - max_d x_t[d]) for every valid frame, in parallel
//   k_rec   one workgroup per (sequence, direction): the alpha recursion of
//           Algorithm 1 and the mirrored beta recursion, time loop on device,
//           the current vector in LDS, arcs in registers or streamed as
//           sliced-ELL records, leaky-HMM mixing and per-frame rescaling fused,
//           scaled trellis rows and per-frame normalisers spilled to HBM; the
//           workgroup that finishes a sequence second then runs the scan: fp64
//           prefix sums of the log normalisers, log Z, per-frame occupancy
//           scale, objective and status
//   k_occ   pdf occupancies of Eq. 3 for every frame in parallel and the
//           gradient write
//
// Scaled quantities: alpha'_t = ahat_t * exp(sum_{tau<=t} log n_tau) * (frame
// maxima), likewise beta; the frame maxima cancel in the occupancies and are
// added back into log Z.
#include "kernels.h"

#include <algorithm>

namespace lfmmi {
namespace {

template <typename Real>
__device__ __forceinline__ Real wave_sum(Real v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Element of an LDS array addressed by the record's index * 4 field.
template <typename Real>
__device__ __forceinline__ Real lds_at(const Real* base, uint32_t index4)
{
    return *reinterpret_cast<const Real*>(reinterpret_cast<const char*>(base) +
                                          index4 * (uint32_t)(sizeof(Real) / 4));
}

// ---------------------------------------------------------------------------
// Emission: one wave per frame row. A row holding NaN or +inf (or nothing but
// -inf) is flagged by a NaN row maximum and an all-zero emission row.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_emit(FbParams p)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int b = p.order[2 * (p.seq_first + blockIdx.y)] >> 1;
    if (blockIdx.x == 0 && threadIdx.x == 0) p.done[b] = 0;  // see k_rec
    if (t >= p.T) return;
    const size_t at = ((size_t)b * p.T + t) * p.P;
    if (t >= p.seqs[b].T) {  // a padding frame: its gradient row is zero
        if (!p.accumulate)
            for (int d = lane; d < p.P; d += 64) p.grad[at + d] = 0.f;
        return;
    }
    if (p.emis_ready) return;  // this frame's emission row and maximum are there already
    const float* x = p.logits + at;
    float* e = p.emis + at;
    float m = -INFINITY;
    bool bad = false;
    for (int d = lane; d < p.P; d += 64) {
        const float v = x[d];
        bad |= !(v == v);
        m = fmaxf(m, v);
    }
    m = wave_max(m);
    bad = __any(bad) || !(fabsf(m) < INFINITY);
    for (int d = lane; d < p.P; d += 64) e[d] = bad ? 0.f : expf(x[d] - m);
    if (lane == 0) p.rowmax[(size_t)b * p.T + t] = bad ? __builtin_nanf("") : m;
}

// ---------------------------------------------------------------------------
// Recursion. Direction 0 is alpha (rows = to-states), direction 1 is beta
// (rows = from-states); both run v <- leak(M v) with
//   leak(v) = v + eps * (a . v) * b     (alpha: a = 1, b = pi; beta: a = pi, b = 1)
// and store vhat = leak(v) / n, n = sum(v).
// ---------------------------------------------------------------------------

// Byte offset of a record's emission value inside a Y buffer: the upper half of
// its key. Plain rows: 4 * pdf. Rows replicated 32 times, so that lane l always
// reads bank l % 32 (conflict-free; small pdf counts only): 128 * pdf + 4 * (l % 32),
// which the upload writes into the device copy of lane l's records.
__device__ __forceinline__ uint32_t y_offset(uint32_t key) { return key >> 16; }

__device__ __forceinline__ float lds_f32(const float* base, uint32_t byte_off)
{
    return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}

// Arc records on the device: the records of slots 2q and 2q + 1 of a lane lie side
// by side, {key, w, key, w}, pair q of lane l at [q * 64 + l] (a 16-byte load per
// lane streams from L2 at twice the rate of an 8-byte one); slices start at even
// slots. The per-arc leak factors are paired up the same way.
__device__ __forceinline__ const uint4* rec_pairs(const FbParams& p, const OrdDesc& od, const int lane)
{
    return reinterpret_cast<const uint4*>(p.g.recs) + (size_t)(od.rec_at >> 1) * 64 + lane;
}
__device__ __forceinline__ const float2* wb_pairs(const FbParams& p, const OrdDesc& od, const int lane)
{
    return reinterpret_cast<const float2*>(p.g.wb) + (size_t)(od.rec_at >> 1) * 64 + lane;
}
__device__ __forceinline__ uint2 rec_lo(const uint4 r) { return make_uint2(r.x, r.y); }
__device__ __forceinline__ uint2 rec_hi(const uint4 r) { return make_uint2(r.z, r.w); }

// The recursion of one (sequence, direction).
//
// Real   float when every state of the graph is final (denominator-like: the
//        scaled vectors stay within fp32 range), double otherwise (left-to-right
//        numerator graphs, where the states that matter can hold a fraction of
//        the frame's mass far below 1e-38).
//        Arc records are streamed from global memory / L2 every frame here;
//        RecRegs below keeps them in registers.
// YREP   emission row replicated across banks.
// HAS_WB the leak target differs per state, so every arc carries w * b[from].
// HUBS   the graph has hub slices (64 lanes that share the arcs of lane 0's row).
//
// Normalisation is lazy: LDS and the trellis hold the raw v_t = M vhat'_{t-1};
// the consumer of v_t applies vhat'_t = v_t / n_t + (eps * s_t / n_t) * b with
// n_t = sum(v_t), s_t = a . v_t, which every lane derives from the 16 wave
// partials after the single barrier of the step. For an arc into row j:
//   v_{t+1}[j] = (1/n_t) * sum w e v_t[from] + (eps s_t / n_t) * sum (w b[from]) e
template <typename Real, bool YREP, bool HAS_WB, int NT, bool HUBS>
__device__ __forceinline__ void rec_run(const FbParams& p, const SeqDesc& sd, const OrdDesc& od,
                                        const int b, const int dir, unsigned char* lds_raw)
{
    // registers that carry the next emission row across a step: enough for a
    // replicated 84-pdf row at the full workgroup size
    constexpr int kYRegs = NT >= 1024 ? 3 : 6;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x;
    const int nwaves = nthreads >> 6;
    const int T = sd.T;
    const int P = p.P;
    const int rows = od.num_slices * 64;
    const int ylen = YREP ? P * 32 : P;           // floats of one emission buffer
    const int ypad = (ylen + 63) & ~63;

    Real* X0 = reinterpret_cast<Real*>(lds_raw);
    Real* X1 = X0 + p.lds_rows;
    Real* part = X1 + p.lds_rows;  // [2][16][2]
    float* Y0 = reinterpret_cast<float*>(part + 64);
    float* Y1 = Y0 + ypad;

    Real* trel = static_cast<Real*>(dir == 0 ? p.alpha : p.beta) +
                 (dir == 0 ? sd.alpha_at : sd.beta_at);
    Real* scalN = static_cast<Real*>(p.scal) + (size_t)(dir * 2) * p.scal_total + sd.scal_at;
    Real* scalS = scalN + p.scal_total;
    const uint4* recs = rec_pairs(p, od, lane);
    const float2* wbp = wb_pairs(p, od, lane);
    const int32_t* so = p.g.slice_off + od.slice_off_at;
    const int32_t* hub = p.g.slice_hub + od.slice_off_at;
    const Real eps = (Real)p.leak;
    const Real bconst = (Real)od.b_const;

    int s0 = 0, s1 = 0;
    if (wave < od.num_waves) {
        s0 = p.g.wave_first[od.wave_first_at + wave];
        s1 = p.g.wave_first[od.wave_first_at + wave + 1];
    }
    const size_t erow0 = (size_t)b * p.T;
    // which of the wave's slices are hub slices: bits for its first 64, a load beyond
    uint64_t hub_bits = 0;
    if (HUBS)
        for (int sl = s0; sl < s1 && sl - s0 < 64; ++sl)
            if (hub[sl]) hub_bits |= (uint64_t)1 << (sl - s0);
    auto hub_at = [&](const int sl) {
        return sl - s0 < 64 ? ((hub_bits >> (sl - s0)) & 1) != 0 : hub[sl] != 0;
    };

    if (tid < 64) part[tid] = 0;  // partials of waves that do not exist stay 0
    __syncthreads();

    // ---- step 0: v_0 = init
    {
        Real n = 0, s = 0;
        const int ti = dir == 0 ? 0 : T;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            const Real v = (Real)p.g.vinit[od.vec_at + row];
            X0[row] = v;
            trel[(size_t)ti * rows + row] = v;
            n += v;
            s += (Real)p.g.va[od.vec_at + row] * v;
        }
        n = wave_sum(n);
        s = wave_sum(s);
        if (lane == 0) { part[wave * 2] = n; part[wave * 2 + 1] = s; }
        if (T > 0) {
            const int fr = dir == 0 ? 0 : T - 1;
            const float* e = p.emis + (erow0 + fr) * P;
            for (int q = tid; q < ylen; q += nthreads) Y0[q] = e[YREP ? q >> 5 : q];
        }
        __syncthreads();
    }

    // ---- steps 1..T
    for (int k = 1; k <= T; ++k) {
        const Real* Xc = (k & 1) ? X0 : X1;
        Real* Xn = (k & 1) ? X1 : X0;
        const float* Yc = (k & 1) ? Y0 : Y1;
        float* Yn = (k & 1) ? Y1 : Y0;
        const Real* partc = part + ((k & 1) ? 0 : 32);
        Real* partn = part + ((k & 1) ? 32 : 0);

        // emission row of the next step, issued early
        float yreg[kYRegs];
        const bool more = k < T;
        const int frn = dir == 0 ? k : T - k - 1;
        const float* en = p.emis + (erow0 + (more ? frn : 0)) * P;
#pragma unroll
        for (int i = 0; i < kYRegs; ++i) {
            const int q = tid + i * nthreads;
            yreg[i] = (more && q < ylen) ? en[YREP ? q >> 5 : q] : 0.f;
        }

        // scalars of the previous step from the wave partials
        Real N = 0, Sd = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { N += partc[w * 2]; Sd += partc[w * 2 + 1]; }
        const Real inv = N > 0 ? (Real)1 / N : (Real)0;
        const Real c = eps * Sd * inv;
        const Real cb = HAS_WB ? c : c * bconst;
        {
            const int tp = dir == 0 ? k - 1 : T - k + 1;
            if (tid == 0) { scalN[tp] = N; scalS[tp] = Sd; }
        }
        const int ti = dir == 0 ? k : T - k;
        Real* tr = trel + (size_t)ti * rows;

        Real n = 0, s = 0;
        {
            for (int sl = s0; sl < s1; ++sl) {
                const int o0 = so[sl], o1 = so[sl + 1] - od.closing;  // without the closing slot
                const uint4* rp = recs + (size_t)(o0 >> 1) * 64;
                const float2* wp = wbp + (size_t)(o0 >> 1) * 64;
                Real acc1 = 0, acc2 = 0;
                auto slot = [&](const uint2 r, const float wbv) {
                    const float e = lds_f32(Yc, y_offset(r.x));
                    const Real x = lds_at(Xc, r.x & 0xffffu);
                    const float t = __uint_as_float(r.y) * e;
                    acc1 += (Real)t * x;
                    acc2 += HAS_WB ? (Real)(wbv * e) : (Real)t;
                };
                int i = o0;
                for (; i + 4 <= o1; i += 4) {
                    const uint4 r0 = rp[0], r1 = rp[64];
                    float2 w0 = make_float2(0.f, 0.f), w1 = w0;
                    if (HAS_WB) {
                        w0 = wp[0];
                        w1 = wp[64];
                    }
                    rp += 128;
                    wp += 128;
                    slot(rec_lo(r0), w0.x);
                    slot(rec_hi(r0), w0.y);
                    slot(rec_lo(r1), w1.x);
                    slot(rec_hi(r1), w1.y);
                }
                // the closing slot (the second half of the slice's last pair: widths are
                // even) holds the row's leak-dot weight
                uint32_t closing_w = 0;
                for (; i < o1; i += 2) {
                    const uint4 r = rp[0];
                    const float2 w = HAS_WB ? wp[0] : make_float2(0.f, 0.f);
                    rp += 64;
                    wp += 64;
                    slot(rec_lo(r), w.x);
                    if (i + 1 < o1) slot(rec_hi(r), w.y);
                    else closing_w = r.w;
                }
                const int row = sl * 64 + lane;
                const bool hub_slice = HUBS && hub_at(sl);  // wave-uniform
                if (hub_slice) {  // its 64 lanes hold the arcs of lane 0's row
                    acc1 = wave_sum(acc1);
                    acc2 = wave_sum(acc2);
                }
                Real v = inv * acc1 + cb * acc2;
                if (hub_slice && lane != 0) v = 0;
                Xn[row] = v;
                tr[row] = v;
                n += v;
                if (HAS_WB) s += (Real)__uint_as_float(closing_w) * v;
            }
        }
        n = wave_sum(n);
        s = HAS_WB ? wave_sum(s) : (Real)od.a_const * n;  // one weight for all rows
        if (lane == 0) { partn[wave * 2] = n; partn[wave * 2 + 1] = s; }
        if (more) {
#pragma unroll
            for (int i = 0; i < kYRegs; ++i) {
                const int q = tid + i * nthreads;
                if (q < ylen) Yn[q] = yreg[i];
            }
            for (int q = tid + kYRegs * nthreads; q < ylen; q += nthreads)
                Yn[q] = en[YREP ? q >> 5 : q];
        }
        __syncthreads();
    }

    // ---- last scalars and the closing dot product:
    // alpha side sum_j f[j] ahat'_T[j], beta side sum_i pi[i] bhat'_0[i]
    {
        const Real* Xc = (T & 1) ? X1 : X0;
        const Real* partc = part + ((T & 1) ? 32 : 0);
        Real N = 0, Sd = 0;
        for (int w = 0; w < nwaves; ++w) { N += partc[w * 2]; Sd += partc[w * 2 + 1]; }
        const Real inv = N > 0 ? (Real)1 / N : (Real)0;
        const Real c = eps * Sd * inv;
        const int tp = dir == 0 ? T : 0;
        if (tid == 0) { scalN[tp] = N; scalS[tp] = Sd; }
        Real z = 0;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            const Real v = Xc[row] * inv + c * (Real)p.g.vb[od.vec_at + row];
            z += (Real)p.g.vfin[od.vec_at + row] * v;
        }
        z = wave_sum(z);
        __syncthreads();  // every wave has read its partials
        if (lane == 0) part[wave] = z;
        __syncthreads();
        if (tid == 0) {
            Real Z = 0;
            for (int w = 0; w < nwaves; ++w) Z += part[w];
            static_cast<Real*>(p.zfin)[(size_t)dir * p.B + b] = Z;
        }
    }
}

// ---------------------------------------------------------------------------
// Wave-level sums on the DPP cross-lane path (no LDS traffic).
// ---------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v)
{
    // lanes of rows outside ROW_MASK, and lanes whose source is out of range, add 0
    const int moved =
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return v + __int_as_float(moved);
}

// fp64: the two halves of the value travel separately
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v)
{
    const long long bits = __double_as_longlong(v);
    // (with every row written the old value is dead: bound_ctrl lets the compiler drop the
    // two moves that would zero it first)
    constexpr bool kAll = ROW_MASK == 0xf;
    const int lo = __builtin_amdgcn_update_dpp(0, (int)bits, CTRL, ROW_MASK, 0xf, kAll);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), CTRL, ROW_MASK, 0xf, kAll);
    return v + __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// After this every lane holds the sum over its row of 16 lanes.
template <typename Real>
__device__ __forceinline__ Real row16_allsum(Real v)
{
    v = dpp_add<0xB1, 0xf>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xf>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141, 0xf>(v);  // row_half_mirror
    v = dpp_add<0x140, 0xf>(v);  // row_mirror
    return v;
}

// The value lane `l` holds, as a wave-uniform value.
__device__ __forceinline__ float lane_value(float v, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ double lane_value(double v, int l)
{
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)bits, l);
    const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), l);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Sum over the 64 lanes, returned as a wave-uniform value.
template <typename Real>
__device__ __forceinline__ Real wave_sum_uniform(Real v)
{
    v = row16_allsum(v);
    v = dpp_add<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
    return lane_value(v, 63);
}

// Wave sums of a and b at once: a 32-lane swap puts a[l] + a[l + 32] in the lower
// half-wave and b[l] + b[l + 32] in the upper one, five DPP steps finish both.
// Lane 31 returns the sum of a, lane 63 the sum of b (other lanes: partial sums).
__device__ __forceinline__ float half_wave_sums(float a, float b)
{
    // lanes 0-31 of [0] keep a, lanes 32-63 of [0] take b's lanes 0-31; [1] the rest
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b),
                                                     false, false);
    float v = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    v = row16_allsum(v);
    return dpp_add<0x142, 0xa>(v);  // row_bcast:15 into rows 1 and 3
}
__device__ __forceinline__ double half_wave_sums(double a, double b)
{
    const long long ab = __double_as_longlong(a), bb = __double_as_longlong(b);
    const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)ab, (unsigned)bb, false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)(ab >> 32), (unsigned)(bb >> 32),
                                                     false, false);
    double v = __longlong_as_double(((long long)hi[0] << 32) | lo[0]) +
               __longlong_as_double(((long long)hi[1] << 32) | lo[1]);
    v = row16_allsum(v);
    return dpp_add<0x142, 0xa>(v);
}

// Lane 63 returns the sum over the wave (other lanes: partial sums).
template <typename Real>
__device__ __forceinline__ Real wave_sum_lane63(Real v)
{
    v = row16_allsum(v);
    v = dpp_add<0x142, 0xa>(v);     // row_bcast:15 into rows 1 and 3
    return dpp_add<0x143, 0xc>(v);  // row_bcast:31 into rows 2 and 3
}

// ---------------------------------------------------------------------------
// The recursion with the wave's arc records in registers (graphs whose waves
// own at most NSLOT slots; state values fp32 or fp64). Fixed LDS map, so that the buffer of the
// current parity is an immediate offset on every LDS instruction:
//   [0, 32K) X0   [32K, 64K) X1   [64K, 96K) Y0   [96K, 128K) Y1   [128K, ...) partials
// The last word of each Y buffer is 0: closing slots read it as their emission,
// so that the slot loop needs no special case for them.
// ---------------------------------------------------------------------------
constexpr uint32_t kRegX1 = 32768, kRegY0 = 65536, kRegY1 = 98304, kRegPart = 131072;
constexpr uint32_t kRegYZero = 32764;  // byte offset of the zero word inside a Y buffer

__host__ __device__ constexpr size_t reg_lds_bytes() { return kRegPart + 3 * 32 * sizeof(double); }

// LDS access by absolute byte address (the kernel's dynamic LDS starts at 0: it
// declares no static LDS), so that the address register goes straight into the
// ds instruction and constant parts fold into its immediate offset.
typedef __attribute__((address_space(3))) float lds_float_t;
__device__ __forceinline__ float lds_ld(uint32_t addr)
{
    return *reinterpret_cast<const lds_float_t*>(static_cast<uintptr_t>(addr));
}
__device__ __forceinline__ void lds_st(uint32_t addr, float v)
{
    *reinterpret_cast<lds_float_t*>(static_cast<uintptr_t>(addr)) = v;
}
typedef __attribute__((address_space(3))) double lds_double_t;
__device__ __forceinline__ void lds_st(uint32_t addr, double v)
{
    *reinterpret_cast<lds_double_t*>(static_cast<uintptr_t>(addr)) = v;
}
template <typename Real>
__device__ __forceinline__ Real lds_ldr(uint32_t addr)
{
    if constexpr (sizeof(Real) == 8)
        return *reinterpret_cast<const lds_double_t*>(static_cast<uintptr_t>(addr));
    else
        return *reinterpret_cast<const lds_float_t*>(static_cast<uintptr_t>(addr));
}

// Phase timers (builds with -DLFMMI_PHASE_TIMERS only; the library as shipped carries
// none of this). k_occ_planes: thread 0 of every workgroup adds the clocks between two
// marks to a counter per phase. Register-resident k_rec: every wave keeps the clocks of
// the four phases of a step in scalar registers and adds them to the counters of its
// wave number when its sequence is done. lfmmi_phase_timers_read() copies them out.
#ifdef LFMMI_PHASE_TIMERS
__device__ unsigned long long g_phase_clocks[16];
__device__ unsigned long long g_rec_clocks[16 * 4 + 1];  // [wave][phase], steps
#define LFMMI_REC_TIMERS unsigned long long rec_clk[4] = {0, 0, 0, 0}, rec_last = 0;
#define LFMMI_REC_BEGIN rec_last = __builtin_amdgcn_s_memtime();
#define LFMMI_REC_MARK(i)                                                  \
    {                                                                      \
        const unsigned long long mark_now_ = __builtin_amdgcn_s_memtime(); \
        rec_clk[i] += mark_now_ - rec_last;                                \
        rec_last = mark_now_;                                              \
    }
#define LFMMI_REC_END(wave, lane, steps)                                              \
    if ((lane) == 0 && (wave) < 16) {                                                 \
        for (int q_ = 0; q_ < 4; ++q_) atomicAdd(&g_rec_clocks[(wave) * 4 + q_], rec_clk[q_]); \
        if ((wave) == 0) atomicAdd(&g_rec_clocks[64], (unsigned long long)(steps));   \
    }
#define LFMMI_MARK_BEGIN unsigned long long mark_last_ = __builtin_amdgcn_s_memtime();
#define LFMMI_MARK(i)                                                              \
    {                                                                              \
        const unsigned long long mark_now_ = __builtin_amdgcn_s_memtime();         \
        if (threadIdx.x == 0) atomicAdd(&g_phase_clocks[i], mark_now_ - mark_last_); \
        mark_last_ = mark_now_;                                                    \
    }
#define LFMMI_COUNT(i) \
    if (threadIdx.x == 0) atomicAdd(&g_phase_clocks[i], 1ull);
#else
#define LFMMI_REC_TIMERS
#define LFMMI_REC_BEGIN
#define LFMMI_REC_MARK(i)
#define LFMMI_REC_END(wave, lane, steps)
#define LFMMI_MARK_BEGIN
#define LFMMI_MARK(i)
#define LFMMI_COUNT(i)
#endif

// Emission staging passes of the variant for workgroups of up to NT threads.
__host__ __device__ constexpr int stage_passes(bool yrep, int nt)
{
    return yrep ? (nt >= 1024 ? 2 : (nt >= 768 ? 3 : 4)) : (nt >= 1024 ? 3 : (nt >= 768 ? 4 : 6));
}

// HYBRID: a wave keeps in registers only the first of its slices that fit NSLOT
// slots and streams the records of the others from L2 every frame (graphs too
// large for the registers: less record traffic than streaming everything).
// BIG: state vectors of 48 KB and emission rows of 16 KB (graphs of up to 12288
// states) instead of 32 KB each.
// HUBS: the graph has hub slices (64 lanes that share one row's arcs, added up where
// the slice ends); variants without it carry none of that code.
template <typename Real, bool YREP, bool HAS_WB, int NSLOT, int NT, bool HYBRID = false,
          bool BIG = false, bool HUBS = false>
struct RecRegs {
    static_assert(!HYBRID || (!HAS_WB && sizeof(Real) == 4), "hybrid: fp32, constant leak weights");
    static_assert(!BIG || (HYBRID && !YREP), "the large map: hybrid, plain emission rows");
    // this variant's LDS map (the names hide the 32 KB map's constants)
    static constexpr uint32_t kRegX1 = BIG ? 49152u : lfmmi::kRegX1;
    static constexpr uint32_t kRegY0 = BIG ? 98304u : lfmmi::kRegY0;
    static constexpr uint32_t kRegY1 = BIG ? 114688u : lfmmi::kRegY1;
    static constexpr uint32_t kRegYZero = BIG ? 16380u : lfmmi::kRegYZero;
    static_assert(lfmmi::kRegPart == 131072u, "both maps end where the partial sums begin");
    static constexpr uint32_t kRB = sizeof(Real);  // bytes of a state value
    // Emission staging. Replicated rows (YREP): a thread writes four of the 32
    // copies of one value with one 16-byte store, kYPass passes of NT threads
    // cover 8 * P <= kYPass * NT quads. Plain rows: one value per thread and pass.
    static constexpr int kYPass = stage_passes(YREP, NT);
    static constexpr int kPrefetch = NT >= 1024 ? 2 : (NT >= 768 ? 4 : 6);
    // Slots whose gathers go out at the start of a step, before the partial sums are
    // turned into this step's scalars: with one pair ahead in the slot loop (the depth
    // that measured best) the LDS pipe would run dry during that serial chain, so a
    // second pair is issued there and the loop falls back to one pair ahead.
    static constexpr int kBurst =
        (kPrefetch == 2 && NSLOT >= 8 && NSLOT <= 26 && !HYBRID) ? 4 : kPrefetch;
    static constexpr int kTailSlots = 4;
    // slot before which a step does its global memory work; every wave must get
    // there, also one that leaves the slot loop early
    static constexpr int kStageAt = NSLOT - kTailSlots > 4 ? 4 : 0;
    static_assert(kStageAt % 2 == 0 && (kStageAt == 0 || kStageAt < NSLOT - kTailSlots),
                  "every wave reaches it");
    static_assert(NSLOT % 2 == 0 && kPrefetch % 2 == 0, "slots are handled in pairs");
    static_assert(NSLOT <= 64, "one bit per resident slot in the 64-bit slice-end and hub masks");

    // Packed slots (the hybrid): both addresses of a slot in one register, taken apart
    // again in every step by two instructions; two registers per slot instead of
    // three keep half as many slots again out of the streamed part, where a slot
    // costs its record's way from L2 on top of its gathers.
    static constexpr bool kPacked = HYBRID;
    static_assert(!kPacked || (kRegY0 & 0xffff7fffu) == 0x10000u, "see y_at()");
    uint32_t xa[kPacked ? 1 : NSLOT];  // byte address of the state value inside X0
    // LDS byte address of the emission value in Y0 (absolute); packed: the state
    // value's address in the lower half, the emission value's address less 64 KB
    // in the upper half
    uint32_t ya[NSLOT];
    float wr[NSLOT];     // arc weight; closing slots: the row's leak-dot weight
    float wbr[HAS_WB ? NSLOT : 1];
    float yreg[kYPass];
    uint32_t ysrc[kYPass];  // byte offset of this thread's value inside an emission row
    uint32_t ydst[kYPass];  // byte offset inside a Y buffer it is stored to
    int ypasses;            // passes in which this wave holds any of the row (wave-uniform)
    // hybrid: lane l holds the end (one past the last slot) of the wave's l-th streamed
    // slice; one past the wave's last slot
    int so_tab, stream_end;

    LFMMI_REC_TIMERS
    // per-step pointers, moved by one frame after every step
    const float* e2;  // emission row loaded during this step (used two steps on)
    Real* trow;       // trellis row written by this step
    Real* sN;         // where the scalars of the previous step go
    Real* sS;
    ptrdiff_t estep, tstep, sstep;

    __device__ __forceinline__ uint32_t x_at(const int i) const
    {
        if constexpr (kPacked) return ya[i] & 0xffffu;
        else return xa[i];
    }
    __device__ __forceinline__ uint32_t y_at(const int i) const
    {
        // the upper half of the register below a 1: 64 KB + the stored half
        if constexpr (kPacked) return __builtin_amdgcn_alignbit(1u, ya[i], 16u);
        else return ya[i];
    }

    __device__ __forceinline__ void load_y()
    {
        const char* base = reinterpret_cast<const char*>(e2);
#pragma unroll
        for (int i = 0; i < kYPass; ++i)
            if (i < ypasses) yreg[i] = *reinterpret_cast<const float*>(base + ysrc[i]);
    }

    __device__ __forceinline__ void store_y(const uint32_t ybuf)
    {
#pragma unroll
        for (int i = 0; i < kYPass; ++i)
            if (i < ypasses) {
                if constexpr (YREP) {
                    // four adjacent words from one register: two 2-word stores (the
                    // compiler would spend a register and an instruction per word).
                    // ydst points at the first or the second pair of the quad by the
                    // parity of the pdf, the other pair follows: the 32 lanes of a
                    // half-wave (8 quads of 4 pdfs) then put two words into every bank
                    // per store, not four into every other pair of banks
                    const uint32_t at = ybuf + ydst[i];
                    asm volatile("ds_write2_b32 %0, %2, %2 offset1:1\n\t"
                                 "ds_write2_b32 %1, %2, %2 offset1:1"
                                 :
                                 : "v"(at), "v"(at ^ 8u), "v"(yreg[i])
                                 : "memory");
                } else {
                    lds_st(ybuf + ydst[i], yreg[i]);
                }
            }
    }

    template <int PAR>
    __device__ __forceinline__ void step(const int k, const int T, const int tid, const int lane,
                                         const Real eps, const Real aconst, const Real bconst,
                                         const uint64_t mask, const uint64_t hubmask,
                                         const uint32_t row4_first,
                                         const uint32_t part_at, const int nsl,
                                         const int sl_stream, const int sl_end,
                                         const int first_streamed, const int32_t* so,
                                         const uint64_t hub_bits, const int32_t* hub,
                                         const uint4* recs_uniform)
    {
        LFMMI_REC_BEGIN
        // PAR = k & 1: read X/Y buffer (PAR ? 0 : 1), write buffer (PAR ? 1 : 0)
        constexpr uint32_t xc = PAR ? 0u : kRegX1, xn = PAR ? kRegX1 : 0u;
        // Y addresses in ya[] are absolute addresses inside Y0; Y1 is 32 KB further
        constexpr uint32_t yc = PAR ? 0u : (kRegY1 - kRegY0), yn = PAR ? kRegY1 : kRegY0;
        constexpr uint32_t pc = kRegPart + (PAR ? 0u : 32u * kRB), pn = kRegPart + (PAR ? 32u * kRB : 0u);

        // First the LDS reads this wave waits for: the partial sums of step k - 1
        // (lanes 0-15 fetch the n partials, 16-31 the s partials) and the first
        // gathers. The scalar chain below then runs while the gathers are in flight.
        if constexpr (kPacked) {
            // opaque once a step: the addresses are taken out of the packed registers
            // where they are used, not once and for all before the time loop
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) asm volatile("" : "+v"(ya[i]));
        }
        Real pv = lds_ldr<Real>(pc + (lane & (HAS_WB ? 31 : 15)) * kRB);
        Real xv[kBurst ? kBurst : 1];
        float ev[kBurst ? kBurst : 1];
#pragma unroll
        for (int i = 0; i < kBurst && i < NSLOT; ++i) {
            xv[i] = lds_ldr<Real>(xc + x_at(i));
            ev[i] = lds_ld(yc + y_at(i));
        }
        asm volatile("" ::: "memory");  // nothing else moves ahead of these reads
        // Without per-row leak-dot weights s is a_const * n.
        pv = row16_allsum(pv);
        const Real N = lane_value(pv, 0);
        const Real Sd = HAS_WB ? lane_value(pv, 16) : aconst * N;
        Real inv = 0;
        if (N > 0) {
            if constexpr (sizeof(Real) == 4) {
                inv = __builtin_amdgcn_rcpf(N);
                inv = fmaf(fmaf(-N, inv, 1.f), inv, inv);  // one Newton step
            } else {
                // hardware reciprocal and two Newton steps (N is a sum of probabilities
                // far from the ends of the fp64 range): a third of the instructions of
                // a division, on the critical path of the short numerator steps
                inv = __builtin_amdgcn_rcp((double)N);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
            }
        }
        const Real c = eps * Sd * inv;
        const Real cb = HAS_WB ? c : c * bconst;
        LFMMI_REC_MARK(0)  // head: last step's partial sums into this step's scalars

        // (the leak's accumulator stays fp32 also beside fp64 state values: a few products
        // of fp32 numbers, which only ever meet the leak coefficient)
        Real acc1 = 0, n = 0, s = 0;
        float acc2 = 0;
        uint64_t left = mask;
        int next_close = left ? __builtin_ctzll(left) : 64;
        uint32_t row4 = row4_first;  // byte offset of this lane's row in a state vector
        char* const tr = reinterpret_cast<char*>(trow);
        // Slots go in pairs: slices are an even number of slots wide, so a slice can
        // only end on the second slot of a pair.
#pragma unroll
        for (int i = 0; i < NSLOT; i += 2) {
            // a wave with fewer slots than the variant holds leaves at its last one
            // (tested near the end only, where the counts of one graph differ)
            if (i > 0 && i >= NSLOT - kTailSlots) {
                int count = nsl;
                asm volatile("" : "+s"(count));  // compare here, in a scalar register
                if (i >= count) break;
            }
            // issue priority falls as the wave advances, so that the waves of a SIMD
            // (served oldest first at equal priority) move through the slots together
            if (i == 0) __builtin_amdgcn_s_setprio(2);
            else if (i == (NSLOT / 6) * 2) __builtin_amdgcn_s_setprio(1);
            else if (i == (NSLOT / 3) * 2) __builtin_amdgcn_s_setprio(0);
            if (i == kStageAt) {
                // Global memory work sits here, a few slots in: the loads it waits for
                // were issued a step ago and the last stores long enough ago to be
                // done, so the wait costs nothing. Emission row of step k + 1 (loaded
                // one step ago) into the other Y buffer, then the loads for step k + 2
                // (past the end both repeat the last row), and the scalars of step k - 1.
                store_y(yn);
                load_y();
                if (tid == 0) {
                    *sN = N;
                    *sS = Sd;
                }
            }
            Real x0, x1;
            float e0, e1;
            if constexpr (kPrefetch == 0) {
                x0 = lds_ldr<Real>(xc + x_at(i)); e0 = lds_ld(yc + y_at(i));
                x1 = lds_ldr<Real>(xc + x_at(i + 1)); e1 = lds_ld(yc + y_at(i + 1));
            } else {
                x0 = xv[i % (kBurst ? kBurst : 1)]; e0 = ev[i % (kBurst ? kBurst : 1)];
                x1 = xv[(i + 1) % (kBurst ? kBurst : 1)]; e1 = ev[(i + 1) % (kBurst ? kBurst : 1)];
            }
            // the slots kPrefetch ahead; those of the opening burst are in flight already
            if (kPrefetch > 0 && i + kPrefetch < NSLOT && i + kPrefetch >= kBurst) {
                constexpr int kp = kPrefetch ? kPrefetch : 1;
                constexpr int kr = kBurst ? kBurst : 1;
                xv[(i + kp) % kr] = lds_ldr<Real>(xc + x_at((i + kp) % NSLOT));
                ev[(i + kp) % kr] = lds_ld(yc + y_at((i + kp) % NSLOT));
                xv[(i + 1 + kp) % kr] = lds_ldr<Real>(xc + x_at((i + 1 + kp) % NSLOT));
                ev[(i + 1 + kp) % kr] = lds_ld(yc + y_at((i + 1 + kp) % NSLOT));
            }
            // one wait for the pair: this names the value loaded last, so the first
            // use of any of the four comes after all of them have arrived
            asm volatile("" : "+v"(x0), "+v"(e0) : "v"(x1), "v"(e1));  // (fp64: register pairs)
            // arc slots; closing and padding slots see e == 0 or w == 0 and add nothing
            const float t0 = wr[i] * e0;
            const float t1 = wr[i + 1] * e1;
            if constexpr (sizeof(Real) == 4) {
                acc1 = fmaf(t0, x0, acc1);
                acc2 = HAS_WB ? fmaf(wbr[HAS_WB ? i : 0], e0, acc2) : acc2 + t0;
                acc1 = fmaf(t1, x1, acc1);
                acc2 = HAS_WB ? fmaf(wbr[HAS_WB ? i + 1 : 0], e1, acc2) : acc2 + t1;
            } else {  // products of the arc weight and the emission stay fp32
                acc1 += (Real)t0 * x0;
                acc2 = HAS_WB ? fmaf(wbr[HAS_WB ? i : 0], e0, acc2) : acc2 + t0;
                acc1 += (Real)t1 * x1;
                acc2 = HAS_WB ? fmaf(wbr[HAS_WB ? i + 1 : 0], e1, acc2) : acc2 + t1;
            }
            if (__builtin_expect(i + 1 == next_close, 0)) {  // wave-uniform: a slice ends
                const bool hub_slice = HUBS && ((hubmask >> (i + 1)) & 1);
                if (hub_slice) {  // its 64 lanes hold the arcs of lane 0's row
                    acc1 = wave_sum_uniform(acc1);
                    acc2 = wave_sum_uniform(acc2);
                }
                Real v = inv * acc1 + cb * (Real)acc2;
                if (hub_slice && lane != 0) v = 0;
                lds_st(xn + row4, v);
                *reinterpret_cast<Real*>(tr + row4) = v;
                n += v;
                if (HAS_WB) s += (Real)wr[i + 1] * v;  // the closing slot's w is a[row]
                acc1 = 0;
                acc2 = 0;
                row4 += 64 * kRB;
                left &= left - 1;
                next_close = left ? __builtin_ctzll(left) : 64;
            }
        }
        if constexpr (HYBRID) {
            // The wave's other slices, their records from L2 (the first of them may
            // have begun in the registers: acc1, acc2). Pairs of slots in a flat
            // sequence, four pairs in registers: two are being used while the two after
            // them load, and the eight gathers of two pairs go out before the first
            // is waited for. Loads past the wave's last pair repeat it (in bounds,
            // never used). Everything that steers the loop is wave-uniform.
            int i = first_streamed;  // even
            Real a1 = acc1, a2 = (Real)acc2;
            if (i < stream_end) {
                // pair q of this lane: a wave-uniform base in scalar registers plus a
                // 32-bit byte offset (one vector add per load, no 64-bit arithmetic)
                typedef const __attribute__((address_space(1))) char* global_bytes_t;
                typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                typedef const __attribute__((address_space(1))) u32x4_t* global_u32x4_t;
                const uint64_t rb = reinterpret_cast<uint64_t>(recs_uniform) + (uint64_t)(i >> 1) * 1024u;
                const global_bytes_t rbase = (global_bytes_t)(
                    ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(rb >> 32)) << 32) |
                    (uint32_t)__builtin_amdgcn_readfirstlane((int)rb));
                const uint32_t lane16 = (uint32_t)lane * 16u;
                auto pair_at = [&](const int q) {
                    const u32x4_t v = *(global_u32x4_t)(rbase + ((uint32_t)q * 1024u + lane16));
                    return make_uint4(v.x, v.y, v.z, v.w);
                };
                const int last = ((stream_end - i) >> 1) - 1;  // index of the wave's last pair
                int sl = sl_stream;
                auto slice_end = [&](const int at) {  // one past the last slot of slice `at`
                    if (at >= sl_end) return stream_end;
                    return at - sl_stream < 64 ? __builtin_amdgcn_readlane(so_tab, at - sl_stream)
                                               : so[at + 1];
                };
                int o1 = slice_end(sl);
                auto close = [&]() {
                    const bool hub_slice =
                        HUBS && (sl - sl_stream < 64 ? ((hub_bits >> (sl - sl_stream)) & 1) != 0
                                                     : hub[sl] != 0);
                    if (hub_slice) {
                        a1 = wave_sum_uniform(a1);
                        a2 = wave_sum_uniform(a2);
                    }
                    Real v = inv * a1 + cb * a2;
                    if (hub_slice && lane != 0) v = 0;
                    const uint32_t at = (uint32_t)(sl * 64 + lane) * kRB;
                    lds_st(xn + at, v);
                    *reinterpret_cast<Real*>(tr + at) = v;
                    n += v;
                    a1 = 0;
                    a2 = 0;
                    ++sl;
                    o1 = slice_end(sl);
                };
                // 64 KB + the upper half of the key in one instruction (the upper half
                // below a 1); what else leads to the Y buffer of this parity is a
                // constant that folds into the offset field of the read
                static_assert(kRegY0 >= 0x10000u && yc + kRegY0 - 0x10000u < 0x10000u, "offset field");
                auto y_of = [&](const uint32_t key) {
                    return (yc + kRegY0 - 0x10000u) + __builtin_amdgcn_alignbit(1u, key, 16u);
                };
                auto two_pairs = [&](const uint4 qa, const uint4 qb, const bool b_valid) {
                    float e0 = lds_ld(y_of(qa.x));
                    Real x0 = lds_ldr<Real>(xc + (qa.x & 0xffffu));
                    float e1 = lds_ld(y_of(qa.z));
                    Real x1 = lds_ldr<Real>(xc + (qa.z & 0xffffu));
                    float e2 = lds_ld(y_of(qb.x));
                    Real x2 = lds_ldr<Real>(xc + (qb.x & 0xffffu));
                    float e3 = lds_ld(y_of(qb.z));
                    Real x3 = lds_ldr<Real>(xc + (qb.z & 0xffffu));
                    // one wait for the eight: the first use names the value loaded last
                    asm volatile("" : "+v"(x0), "+v"(e0), "+v"(x1), "+v"(e1), "+v"(x2), "+v"(e2)
                                 : "v"(x3), "v"(e3));
                    const float t0 = __uint_as_float(qa.y) * e0, t1 = __uint_as_float(qa.w) * e1;
                    a1 = fmaf(t0, x0, a1);
                    a2 += t0;
                    a1 = fmaf(t1, x1, a1);
                    a2 += t1;
                    i += 2;
                    if (i == o1) close();
                    if (b_valid) {
                        const float t2 = __uint_as_float(qb.y) * e2, t3 = __uint_as_float(qb.w) * e3;
                        a1 = fmaf(t2, x2, a1);
                        a2 += t2;
                        a1 = fmaf(t3, x3, a1);
                        a2 += t3;
                        i += 2;
                        if (i == o1) close();
                    }
                };
                uint4 q0 = pair_at(0);
                uint4 q1 = pair_at(min(1, last));
                uint4 q2 = pair_at(min(2, last));
                uint4 q3 = pair_at(min(3, last));
                for (int pr = 0; pr <= last; pr += 4) {
                    two_pairs(q0, q1, pr + 1 <= last);
                    q0 = pair_at(min(pr + 4, last));
                    q1 = pair_at(min(pr + 5, last));
                    if (pr + 2 <= last) two_pairs(q2, q3, pr + 3 <= last);
                    q2 = pair_at(min(pr + 6, last));
                    q3 = pair_at(min(pr + 7, last));
                }
            }
        }
        LFMMI_REC_MARK(1)  // the slots
        __builtin_amdgcn_s_setprio(3);  // the serial end of this step and start of the next
        if constexpr (HAS_WB) {
            // both wave sums in one reduction: lane 31 ends up with n, lane 63 with s
            const Real ns = half_wave_sums(n, s);
            if ((lane & 31) == 31) lds_st(pn + part_at, ns);
        } else {
            const Real ns = wave_sum_lane63(n);
            if (lane == 63) lds_st(pn + part_at, ns);
        }
        if (k + 2 < T) e2 += estep;
        trow += tstep;
        sN += sstep;
        sS += sstep;
        LFMMI_REC_MARK(2)  // tail: wave sum, partial sum to LDS
        __syncthreads();
        LFMMI_REC_MARK(3)  // wait for the other waves
    }

    // A step for a wave that owns at most one slice of at most kLeanSlots slots (the
    // per-utterance numerator graphs: a few hundred states, two or three arcs into each):
    // the same protocol as step() - LDS map, partial sums, one barrier - and the same
    // arithmetic in the same order, so the waves of a workgroup may take either (which one
    // depends on the wave's own slice only); but straight-line: all gathers at once, one close, no
    // slice masks, slot counts or priorities. Such steps are bound by the instructions a
    // wave issues, not by LDS. a_row: the row's leak-dot weight (the closing slot's w).
    static constexpr int kLeanSlots = 4;
    template <int PAR>
    __device__ __forceinline__ void step_lean(const int k, const int T, const int tid, const int lane,
                                              const Real eps, const Real aconst, const Real bconst,
                                              const bool owns, const float a_row,
                                              const uint32_t row4_first, const uint32_t part_at)
    {
        LFMMI_REC_BEGIN
        constexpr uint32_t xc = PAR ? 0u : kRegX1, xn = PAR ? kRegX1 : 0u;
        constexpr uint32_t yc = PAR ? 0u : (kRegY1 - kRegY0), yn = PAR ? kRegY1 : kRegY0;
        constexpr uint32_t pc = kRegPart + (PAR ? 0u : 32u * kRB), pn = kRegPart + (PAR ? 32u * kRB : 0u);
        Real pv = lds_ldr<Real>(pc + (lane & (HAS_WB ? 31 : 15)) * kRB);
        Real xv[kLeanSlots];
        float ev[kLeanSlots];
#pragma unroll
        for (int i = 0; i < kLeanSlots; ++i) {
            xv[i] = lds_ldr<Real>(xc + x_at(i));
            ev[i] = lds_ld(yc + y_at(i));
        }
        asm volatile("" ::: "memory");  // nothing else moves ahead of these reads
        pv = row16_allsum(pv);
        const Real N = lane_value(pv, 0);
        const Real Sd = HAS_WB ? lane_value(pv, 16) : aconst * N;
        Real inv = 0;
        if (N > 0) {
            if constexpr (sizeof(Real) == 4) {
                inv = __builtin_amdgcn_rcpf(N);
                inv = fmaf(fmaf(-N, inv, 1.f), inv, inv);
            } else {
                inv = __builtin_amdgcn_rcp((double)N);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
            }
        }
        const Real c = eps * Sd * inv;
        const Real cb = HAS_WB ? c : c * bconst;
        LFMMI_REC_MARK(0)
        store_y(yn);
        load_y();
        if (tid == 0) {
            *sN = N;
            *sS = Sd;
        }
        Real acc1 = 0;
        float acc2 = 0;
#pragma unroll
        for (int i = 0; i < kLeanSlots; ++i) {
            const float t = wr[i] * ev[i];
            if constexpr (sizeof(Real) == 4) acc1 = fmaf(t, xv[i], acc1);
            else acc1 += (Real)t * xv[i];
            acc2 = HAS_WB ? fmaf(wbr[HAS_WB ? i : 0], ev[i], acc2) : acc2 + t;
        }
        Real n = 0, s = 0;
        if (owns) {
            const Real v = inv * acc1 + cb * (Real)acc2;
            lds_st(xn + row4_first, v);
            *reinterpret_cast<Real*>(reinterpret_cast<char*>(trow) + row4_first) = v;
            n = v;
            if (HAS_WB) s = (Real)a_row * v;
        }
        LFMMI_REC_MARK(1)
        if constexpr (HAS_WB) {
            const Real ns = half_wave_sums(n, s);
            if ((lane & 31) == 31) lds_st(pn + part_at, ns);
        } else {
            const Real ns = wave_sum_lane63(n);
            if (lane == 63) lds_st(pn + part_at, ns);
        }
        if (k + 2 < T) e2 += estep;
        trow += tstep;
        sN += sstep;
        sS += sstep;
        LFMMI_REC_MARK(2)
        __syncthreads();
        LFMMI_REC_MARK(3)
    }

    __device__ __forceinline__ void run(const FbParams& p, const SeqDesc& sd, const OrdDesc& od,
                                        const int b, const int dir, unsigned char* lds)
    {
        const int tid = threadIdx.x;
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int nthreads = blockDim.x;
        const int T = sd.T;
        const int P = p.P;
        const int rows = od.num_slices * 64;
        Real* trel = static_cast<Real*>(dir == 0 ? p.alpha : p.beta) +
                     (dir == 0 ? sd.alpha_at : sd.beta_at);
        Real* scalN = static_cast<Real*>(p.scal) + (size_t)(dir * 2) * p.scal_total + sd.scal_at;
        Real* scalS = scalN + p.scal_total;
        const uint4* recs = rec_pairs(p, od, lane);
        // one record: slot s of this lane is the (s & 1)-th half of pair s >> 1
        const uint2* rec1 = reinterpret_cast<const uint2*>(recs);
        const float* wb1 = reinterpret_cast<const float*>(wb_pairs(p, od, lane));
        const int32_t* so = p.g.slice_off + od.slice_off_at;
        const Real eps = (Real)p.leak;
        const Real aconst = (Real)od.a_const;
        const Real bconst = (Real)od.b_const;
        const float* erows = p.emis + (size_t)b * p.T * P;  // this sequence's emission rows

        const int32_t* hub = p.g.slice_hub + od.slice_off_at;
        int s0 = 0, s1 = 0;
        uint64_t mask = 0, hubmask = 0;
        if (wave < od.num_waves) {
            s0 = p.g.wave_first[od.wave_first_at + wave];
            s1 = p.g.wave_first[od.wave_first_at + wave + 1];
            mask = p.g.wave_mask[od.mask_at + wave];
            hubmask = p.g.wave_hub[od.mask_at + wave];
        }
        const int first = so[s0];
        uint64_t hub_bits = 0;  // hub slices among the streamed ones, from sl_stream on
        int sl_stream = s1;  // first slice with streamed records
        int nsl = so[s1] - first;
        if constexpr (HYBRID) {
            // resident: the wave's first NSLOT slots; the slices that end there make
            // the mask, the one that straddles the limit is finished from L2
            nsl = min(nsl, NSLOT);
            mask = 0;
            hubmask = 0;
            sl_stream = s0;
            while (sl_stream < s1 && so[sl_stream + 1] - first <= nsl) {
                const uint64_t bit = (uint64_t)1 << (so[sl_stream + 1] - 1 - first);
                mask |= bit;
                if (HUBS && hub[sl_stream]) hubmask |= bit;
                ++sl_stream;
            }
            if (HUBS)  // bits for the first 64 streamed slices, a load beyond
                for (int sl = sl_stream; sl < s1 && sl - sl_stream < 64; ++sl)
                    if (hub[sl]) hub_bits |= (uint64_t)1 << (sl - sl_stream);
            so_tab = so[max(min(sl_stream + lane, s1 - 1), 0) + 1];
            stream_end = so[s1];
        }
#pragma unroll
        for (int i = 0; i < NSLOT; ++i) {
            const bool on = i < nsl;
            const bool closing = HAS_WB && ((mask >> i) & 1);  // holds a[row], no arc
            const size_t at = (size_t)((first + i) >> 1) * 128 + ((first + i) & 1);
            const uint2 r = on ? rec1[at] : make_uint2(0u, 0u);
            const uint32_t x_addr = (r.x & 0xffffu) * (kRB / 4u);
            const uint32_t y_addr = kRegY0 + ((on && !closing) ? y_offset(r.x) : kRegYZero);
            wr[i] = __uint_as_float(r.y);
            if (HAS_WB) wbr[i] = (on && !closing) ? wb1[at] : 0.f;
            // opaque from here on: the values stay in their registers for the whole
            // time loop instead of being re-derived from the record each frame
            if constexpr (kPacked) {
                ya[i] = x_addr | ((y_addr - 0x10000u) << 16);
                asm volatile("" : "+v"(ya[i]), "+v"(wr[i]));
            } else {
                xa[i] = x_addr;
                ya[i] = y_addr;
                asm volatile("" : "+v"(xa[i]), "+v"(ya[i]), "+v"(wr[i]));
            }
        }
        // emission staging: which value of a row this thread fetches in pass i, and
        // where in a Y buffer it goes
        {
            const int units = YREP ? P * 8 : P;  // 16-byte quads, or single values
            // (a wave whose threads all lie past the row in a pass skips it; single
            // threads past the row repeat the work of an earlier thread)
            ypasses = max(0, (units - wave * 64 + nthreads - 1) / nthreads);
#pragma unroll
            for (int i = 0; i < kYPass; ++i) {
                // threads past the row repeat the work of an earlier thread
                const int q = (tid + i * nthreads) % units;
                ysrc[i] = (uint32_t)(YREP ? q >> 3 : q) * 4u;
                ydst[i] = (uint32_t)q * (YREP ? 16u : 4u) + (YREP ? (uint32_t)((q >> 3) & 1) * 8u : 0u);
            }
        }

        // zero words of the Y buffers, partial slots
        if (tid == 0) {
            lds_st(kRegY0 + kRegYZero, 0.f);
            lds_st(kRegY1 + kRegYZero, 0.f);
        }
        if (tid < 64) lds_st(kRegPart + tid * kRB, (Real)0);
        __syncthreads();

        // ---- step 0: v_0 = init into X0, partials into slot set 0
        {
            Real n = 0, s = 0;
            const int ti = dir == 0 ? 0 : T;
            for (int sl = s0; sl < s1; ++sl) {
                const int row = sl * 64 + lane;
                const Real v = (Real)p.g.vinit[od.vec_at + row];
                lds_st(row * kRB, v);
                trel[(size_t)ti * rows + row] = v;
                n += v;
                s += (Real)p.g.va[od.vec_at + row] * v;
            }
            n = wave_sum_uniform(n);
            s = wave_sum_uniform(s);
            if (lane == 0) {
                lds_st(kRegPart + wave * kRB, n);
                lds_st(kRegPart + (16 + wave) * kRB, s);
            }
            // rows of steps 1 (into Y0 now) and 2 (into registers); frame of step k:
            // FWD k - 1, BWD T - k, kept inside the sequence when T is short
            auto frame_of = [&](int k) {
                const int fr = dir == 0 ? k - 1 : T - k;
                return max(0, min(fr, T - 1));
            };
            if (T > 0) {
                e2 = erows + (size_t)frame_of(1) * P;
                load_y();
                store_y(kRegY0);
                e2 = erows + (size_t)frame_of(2) * P;
                load_y();
                e2 = erows + (size_t)frame_of(3) * P;
            }
            __syncthreads();
        }
        estep = dir == 0 ? (ptrdiff_t)P : -(ptrdiff_t)P;
        tstep = dir == 0 ? (ptrdiff_t)rows : -(ptrdiff_t)rows;
        sstep = dir == 0 ? 1 : -1;
        trow = trel + (size_t)(dir == 0 ? 1 : T - 1) * rows;  // step 1 writes row 1 / T - 1
        sN = scalN + (dir == 0 ? 0 : T);                      // and the scalars of step 0
        sS = scalS + (dir == 0 ? 0 : T);

        const uint32_t row4_first = (uint32_t)(s0 * 64 + lane) * kRB;
        // where this lane's end-of-step sum goes: n of wave w at value w, s at 16 + w
        const uint32_t part_at = ((uint32_t)wave + (HAS_WB && lane >= 32 ? 16u : 0u)) * kRB;
        int k = 1;
        if constexpr (!HYBRID && !HUBS && NSLOT <= 8 && NSLOT >= kLeanSlots) {
            if (s1 - s0 <= 1 && nsl <= kLeanSlots) {  // wave-uniform
                const bool owns = s1 > s0;
                float a_row = 0.f;  // the closing slot is the slice's last
                if (HAS_WB && owns) a_row = nsl == 2 ? wr[1] : wr[kLeanSlots - 1];
                for (; k + 1 <= T; k += 2) {
                    step_lean<1>(k, T, tid, lane, eps, aconst, bconst, owns, a_row, row4_first, part_at);
                    step_lean<0>(k + 1, T, tid, lane, eps, aconst, bconst, owns, a_row, row4_first, part_at);
                }
                if (k <= T)
                    step_lean<1>(k, T, tid, lane, eps, aconst, bconst, owns, a_row, row4_first, part_at);
                k = T + 1;
            }
        }
        for (; k + 1 <= T; k += 2) {
            step<1>(k, T, tid, lane, eps, aconst, bconst, mask, hubmask, row4_first, part_at, nsl,
                    sl_stream, s1, first + nsl, so, hub_bits, hub, rec_pairs(p, od, 0));
            step<0>(k + 1, T, tid, lane, eps, aconst, bconst, mask, hubmask, row4_first, part_at, nsl,
                    sl_stream, s1, first + nsl, so, hub_bits, hub, rec_pairs(p, od, 0));
        }
        if (k <= T) step<1>(k, T, tid, lane, eps, aconst, bconst, mask, hubmask, row4_first, part_at, nsl,
                    sl_stream, s1, first + nsl, so, hub_bits, hub, rec_pairs(p, od, 0));
        LFMMI_REC_END(wave, lane, T)

        // ---- last scalars and the closing dot product
        {
            const uint32_t xc = (T & 1) ? kRegX1 : 0u;
            const uint32_t pc = kRegPart + ((T & 1) ? 32u * kRB : 0u);
            Real pv = lds_ldr<Real>(pc + (lane & (HAS_WB ? 31 : 15)) * kRB);
            pv = row16_allsum(pv);
            const Real N = lane_value(pv, 0);
            const Real Sd = HAS_WB ? lane_value(pv, 16) : aconst * N;
            const Real inv = N > 0 ? (Real)1 / N : (Real)0;
            const Real c = eps * Sd * inv;
            if (tid == 0) {
                const int tp = dir == 0 ? T : 0;
                scalN[tp] = N;
                scalS[tp] = Sd;
            }
            Real z = 0;
            for (int sl = s0; sl < s1; ++sl) {
                const int row = sl * 64 + lane;
                const Real v = lds_ldr<Real>(xc + row * kRB) * inv +
                               c * (Real)p.g.vb[od.vec_at + row];
                z += (Real)p.g.vfin[od.vec_at + row] * v;
            }
            z = wave_sum_uniform(z);
            __syncthreads();  // every wave has read the partials
            if (lane == 0) lds_st(kRegPart + (64 + wave) * kRB, z);
            __syncthreads();
            if (tid == 0) {
                Real Z = 0;
                for (int w = 0; w < (nthreads >> 6); ++w)
                    Z += lds_ldr<Real>(kRegPart + (64 + w) * kRB);
                static_cast<Real*>(p.zfin)[(size_t)dir * p.B + b] = Z;
            }
        }
    }
};

// ---------------------------------------------------------------------------
// The register-resident recursion for graphs whose arcs all take the emission of
// the state they enter (PackedGraph::pdf_by_dst; graphs expanded from HMMs whose
// states emit, Section 4.2): no emission gather per arc.
//   alpha (rows = to-states): the emission is a function of the row,
//       v_t[j] = e_t[pdf_j] * ((1/n) sum_a w_a v[from_a] + (eps s / n) sum_a w_a b[from_a]),
//     one gather per arc and one multiply where a slice ends (normalisation is lazy
//     as in RecRegs; the second sum does not depend on the frame).
//   beta (rows = from-states): the emission is a function of the gathered state, so
//     it is folded into the stored vector: after the barrier that ends a step every
//     lane rewrites its own rows, u[j] = e[pdf_j] * (v[j] / n + eps s / n), a second
//     barrier follows, then v_new[i] = sum_a w_a u[to_a], one gather per arc.
// What is staged per step is the emission per row, EY[row] = e[pdf_row] (thread i
// fetches the values of rows i, i + threads, ... two steps ahead and stores them
// one step ahead), not a replicated emission row.
// LDS map: X0 [0, 32K)  X1 [32K, 64K)  EY0 [64K, 96K)  EY1 [96K, 128K)  partial sums.
// The last value of each X buffer is a zero nobody writes: closing slots gather it
// (rows <= capacity - 64 is checked on the host).
// ---------------------------------------------------------------------------
constexpr int kGroupedPasses = 4;  // rows <= kGroupedPasses * threads in this variant

template <typename Real, bool HAS_WB, int NSLOT, int NT>
struct RecGrouped {
    static constexpr uint32_t kRB = sizeof(Real);
    static constexpr int kYPass = kGroupedPasses;
    static constexpr int kChunk = 4;  // beta: slices whose rows are folded at a time
    static constexpr int kPrefetch = NT >= 1024 ? 2 : 4;  // (twice the depth measured no faster)
    static constexpr int kBurst = (kPrefetch == 2 && NSLOT >= 8) ? 4 : kPrefetch;  // see RecRegs
    static constexpr int kTailSlots = 4;
    static constexpr int kStageAt = NSLOT - kTailSlots > 4 ? 4 : 0;
    static constexpr uint32_t kZeroX = kRegX1 - kRB;  // byte offset of the zero inside an X buffer
    static_assert(NSLOT % 2 == 0 && kPrefetch % 2 == 0, "slots are handled in pairs");
    static_assert(NSLOT <= 64, "one bit per resident slot in the 64-bit slice-end mask");

    uint32_t xa[NSLOT];  // byte address of the gathered state value inside X0
    float wr[NSLOT];     // arc weight; closing slots: the row's leak-dot weight
    float wbr[HAS_WB ? NSLOT : 1];
    float yreg[kYPass];     // emission values of rows tid + i * threads, two steps ahead
    uint32_t ysrc[kYPass];  // byte offset of such a row's pdf inside an emission row
    uint32_t ydst[kYPass];  // byte offset of the row inside an EY buffer
    int ypasses;            // passes in which this wave holds any row (wave-uniform)
    int nslices;            // slices this wave owns (wave-uniform)

    const float* e2;
    Real* trow;
    Real* sN;
    Real* sS;
    ptrdiff_t estep, tstep, sstep;

    __device__ __forceinline__ void load_y()
    {
        const char* base = reinterpret_cast<const char*>(e2);
#pragma unroll
        for (int i = 0; i < kYPass; ++i)
            if (i < ypasses) yreg[i] = *reinterpret_cast<const float*>(base + ysrc[i]);
    }

    __device__ __forceinline__ void store_y(const uint32_t eybuf)
    {
#pragma unroll
        for (int i = 0; i < kYPass; ++i)
            if (i < ypasses) lds_st(eybuf + ydst[i], yreg[i]);
    }

    // DIR 0: alpha, 1: beta. PAR = k & 1 as in RecRegs.
    template <int PAR, int DIR>
    __device__ __forceinline__ void step(const int k, const int T, const int tid, const int lane,
                                         const Real eps, const Real aconst, const Real bconst,
                                         const uint64_t mask, const uint32_t row4_first,
                                         const uint32_t ey_first, const uint32_t part_at,
                                         const int nsl)
    {
        constexpr uint32_t xc = PAR ? 0u : kRegX1, xn = PAR ? kRegX1 : 0u;
        constexpr uint32_t eyc = PAR ? kRegY0 : kRegY1, eyn = PAR ? kRegY1 : kRegY0;
        constexpr uint32_t pc = kRegPart + (PAR ? 0u : 32u * kRB), pn = kRegPart + (PAR ? 32u * kRB : 0u);
        constexpr int kp = kPrefetch, kr = kBurst;

        Real pv = lds_ldr<Real>(pc + (lane & (HAS_WB ? 31 : 15)) * kRB);
        Real xv[kr];
        Real own[DIR == 1 ? kChunk : 1];
        float eown[DIR == 1 ? kChunk : 1];
        float e_close = 0.f;  // alpha: emission of the row whose slice ends next
        if constexpr (DIR == 0) {
#pragma unroll
            for (int i = 0; i < kr && i < NSLOT; ++i) xv[i] = lds_ldr<Real>(xc + xa[i]);
            e_close = lds_ld(eyc + ey_first);
        } else {
            // this lane's own rows of the vector the last step wrote, and their
            // emissions: the first kChunk slices now, with the partial sums
#pragma unroll
            for (int q = 0; q < kChunk; ++q)
                if (q < nslices) {
                    own[q] = lds_ldr<Real>(xc + row4_first + (uint32_t)q * 64u * kRB);
                    eown[q] = lds_ld(eyc + ey_first + (uint32_t)q * 256u);
                }
        }
        asm volatile("" ::: "memory");
        pv = row16_allsum(pv);
        const Real N = lane_value(pv, 0);
        const Real Sd = HAS_WB ? lane_value(pv, 16) : aconst * N;
        Real inv = 0;
        if (N > 0) {
            if constexpr (sizeof(Real) == 4) {
                inv = __builtin_amdgcn_rcpf(N);
                inv = fmaf(fmaf(-N, inv, 1.f), inv, inv);
            } else {
                inv = __builtin_amdgcn_rcp((double)N);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
                inv = fma(fma(-N, inv, (Real)1), inv, inv);
            }
        }
        const Real c = eps * Sd * inv;
        const Real cb = HAS_WB ? c : c * bconst;
        if constexpr (DIR == 1) {
            // fold normalisation, leak and emission into the stored vector, in place
#pragma unroll
            for (int q = 0; q < kChunk; ++q)
                if (q < nslices)
                    lds_st(xc + row4_first + (uint32_t)q * 64u * kRB,
                           (Real)eown[q] * (own[q] * inv + cb));
            for (int q0 = kChunk; q0 < nslices; q0 += kChunk) {  // a wave with many slices
#pragma unroll
                for (int q = 0; q < kChunk; ++q)
                    if (q0 + q < nslices) {
                        own[q] = lds_ldr<Real>(xc + row4_first + (uint32_t)(q0 + q) * 64u * kRB);
                        eown[q] = lds_ld(eyc + ey_first + (uint32_t)(q0 + q) * 256u);
                    }
#pragma unroll
                for (int q = 0; q < kChunk; ++q)
                    if (q0 + q < nslices)
                        lds_st(xc + row4_first + (uint32_t)(q0 + q) * 64u * kRB,
                               (Real)eown[q] * (own[q] * inv + cb));
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kr && i < NSLOT; ++i) xv[i] = lds_ldr<Real>(xc + xa[i]);
            asm volatile("" ::: "memory");
        }

        Real acc1 = 0, acc2 = 0, n = 0, s = 0;
        uint64_t left = mask;
        int next_close = left ? __builtin_ctzll(left) : 64;
        uint32_t row4 = row4_first;  // byte offset of this lane's row in a state vector
        uint32_t ey4 = ey_first;     // ... and in an EY buffer
        char* const tr = reinterpret_cast<char*>(trow);
#pragma unroll
        for (int i = 0; i < NSLOT; i += 2) {
            if (i > 0 && i >= NSLOT - kTailSlots) {
                int count = nsl;
                asm volatile("" : "+s"(count));
                if (i >= count) break;
            }
            if (i == 0) __builtin_amdgcn_s_setprio(2);
            else if (i == (NSLOT / 6) * 2) __builtin_amdgcn_s_setprio(1);
            else if (i == (NSLOT / 3) * 2) __builtin_amdgcn_s_setprio(0);
            if (i == kStageAt) {
                // emission values of step k + 1 (loaded a step ago) into the other EY
                // buffer, the loads for step k + 2, and the scalars of step k - 1
                store_y(eyn);
                load_y();
                if (tid == 0) {
                    *sN = N;
                    *sS = Sd;
                }
            }
            Real x0 = xv[i % kr], x1 = xv[(i + 1) % kr];
            if (i + kp < NSLOT && i + kp >= kr) {  // (the opening burst is in flight already)
                xv[(i + kp) % kr] = lds_ldr<Real>(xc + xa[(i + kp) % NSLOT]);
                xv[(i + 1 + kp) % kr] = lds_ldr<Real>(xc + xa[(i + 1 + kp) % NSLOT]);
            }
            asm volatile("" : "+v"(x0) : "v"(x1));  // one wait for the pair
            if constexpr (sizeof(Real) == 4) {
                acc1 = fmaf(wr[i], x0, acc1);
                acc1 = fmaf(wr[i + 1], x1, acc1);
            } else {
                acc1 += (Real)wr[i] * x0;
                acc1 += (Real)wr[i + 1] * x1;
            }
            if constexpr (DIR == 0)  // the leak's share of the row: frame-independent
                acc2 += HAS_WB ? (Real)(wbr[HAS_WB ? i : 0] + wbr[HAS_WB ? i + 1 : 0])
                               : (Real)(wr[i] + wr[i + 1]);
            if (__builtin_expect(i + 1 == next_close, 0)) {  // wave-uniform: a slice ends
                Real v;
                if constexpr (DIR == 0) v = (Real)e_close * (inv * acc1 + cb * acc2);
                else v = acc1;
                lds_st(xn + row4, v);
                *reinterpret_cast<Real*>(tr + row4) = v;
                n += v;
                if (HAS_WB) s += (Real)wr[i + 1] * v;  // the closing slot's w is a[row]
                acc1 = 0;
                acc2 = 0;
                row4 += 64 * kRB;
                ey4 += 256u;
                left &= left - 1;
                next_close = left ? __builtin_ctzll(left) : 64;
                // (past the wave's last slice this reads a word nobody uses)
                if constexpr (DIR == 0) e_close = lds_ld(eyc + ey4);
            }
        }
        __builtin_amdgcn_s_setprio(3);
        if constexpr (HAS_WB) {
            const Real ns = half_wave_sums(n, s);
            if ((lane & 31) == 31) lds_st(pn + part_at, ns);
        } else {
            const Real ns = wave_sum_lane63(n);
            if (lane == 63) lds_st(pn + part_at, ns);
        }
        if (k + 2 < T) e2 += estep;
        trow += tstep;
        sN += sstep;
        sS += sstep;
        __syncthreads();
    }

    template <int DIR>
    __device__ __forceinline__ void loop(const int T, const int tid, const int lane, const Real eps,
                                         const Real aconst, const Real bconst, const uint64_t mask,
                                         const uint32_t row4_first, const uint32_t ey_first,
                                         const uint32_t part_at, const int nsl)
    {
        int k = 1;
        for (; k + 1 <= T; k += 2) {
            step<1, DIR>(k, T, tid, lane, eps, aconst, bconst, mask, row4_first, ey_first, part_at, nsl);
            step<0, DIR>(k + 1, T, tid, lane, eps, aconst, bconst, mask, row4_first, ey_first, part_at, nsl);
        }
        if (k <= T)
            step<1, DIR>(k, T, tid, lane, eps, aconst, bconst, mask, row4_first, ey_first, part_at, nsl);
    }

    __device__ __forceinline__ void run(const FbParams& p, const SeqDesc& sd, const OrdDesc& od,
                                        const int b, const int dir)
    {
        const int tid = threadIdx.x;
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int nthreads = blockDim.x;
        const int T = sd.T;
        const int P = p.P;
        const int rows = od.num_slices * 64;
        Real* trel = static_cast<Real*>(dir == 0 ? p.alpha : p.beta) +
                     (dir == 0 ? sd.alpha_at : sd.beta_at);
        Real* scalN = static_cast<Real*>(p.scal) + (size_t)(dir * 2) * p.scal_total + sd.scal_at;
        Real* scalS = scalN + p.scal_total;
        const uint2* rec1 = reinterpret_cast<const uint2*>(rec_pairs(p, od, lane));
        const float* wb1 = reinterpret_cast<const float*>(wb_pairs(p, od, lane));
        const int32_t* so = p.g.slice_off + od.slice_off_at;
        const Real eps = (Real)p.leak;
        const Real aconst = (Real)od.a_const;
        const Real bconst = (Real)od.b_const;
        const float* erows = p.emis + (size_t)b * p.T * P;

        int s0 = 0, s1 = 0;
        uint64_t mask = 0;
        if (wave < od.num_waves) {
            s0 = p.g.wave_first[od.wave_first_at + wave];
            s1 = p.g.wave_first[od.wave_first_at + wave + 1];
            mask = p.g.wave_mask[od.mask_at + wave];
        }
        const int first = so[s0];
        const int nsl = so[s1] - first;
        nslices = s1 - s0;
#pragma unroll
        for (int i = 0; i < NSLOT; ++i) {
            const bool on = i < nsl;
            const bool closing = HAS_WB && ((mask >> i) & 1);  // holds a[row], no arc
            const size_t at = (size_t)((first + i) >> 1) * 128 + ((first + i) & 1);
            const uint2 r = on ? rec1[at] : make_uint2(0u, 0u);
            xa[i] = (on && !closing) ? (r.x & 0xffffu) * (kRB / 4u) : kZeroX;
            wr[i] = __uint_as_float(r.y);
            if (HAS_WB) wbr[i] = (on && !closing) ? wb1[at] : 0.f;
            asm volatile("" : "+v"(xa[i]), "+v"(wr[i]));
        }
        // emission staging: row tid + i * threads in pass i (rows <= kYPass * threads is
        // checked on the host; a wave whose threads all lie past the rows skips the pass)
        ypasses = min(kYPass, max(0, (rows - wave * 64 + nthreads - 1) / nthreads));
#pragma unroll
        for (int i = 0; i < kYPass; ++i) {
            const int row = min(tid + i * nthreads, rows - 1);
            ysrc[i] = (uint32_t)p.g.row_pdf[od.vec_at + row] * 4u;
            ydst[i] = (uint32_t)row * 4u;
            yreg[i] = 0.f;
        }
        if (tid == 0) {
            lds_st(kZeroX, (Real)0);
            lds_st(kRegX1 + kZeroX, (Real)0);
        }
        if (tid < 64) lds_st(kRegPart + tid * kRB, (Real)0);
        __syncthreads();

        const uint32_t row4_first = (uint32_t)(s0 * 64 + lane) * kRB;
        const uint32_t ey_first = (uint32_t)(s0 * 64 + lane) * 4u;
        // ---- step 0: v_0 = init into X0, partials into slot set 0
        {
            Real n = 0, s = 0;
            const int ti = dir == 0 ? 0 : T;
            for (int sl = s0; sl < s1; ++sl) {
                const int row = sl * 64 + lane;
                const Real v = (Real)p.g.vinit[od.vec_at + row];
                lds_st(row * kRB, v);
                trel[(size_t)ti * rows + row] = v;
                n += v;
                s += (Real)p.g.va[od.vec_at + row] * v;
            }
            n = wave_sum_uniform(n);
            s = wave_sum_uniform(s);
            if (lane == 0) {
                lds_st(kRegPart + wave * kRB, n);
                lds_st(kRegPart + (16 + wave) * kRB, s);
            }
            auto frame_of = [&](int k) {  // FWD k - 1, BWD T - k, kept inside the sequence
                const int fr = dir == 0 ? k - 1 : T - k;
                return max(0, min(fr, T - 1));
            };
            if (T > 0) {
                e2 = erows + (size_t)frame_of(1) * P;
                load_y();
                store_y(kRegY0);
                e2 = erows + (size_t)frame_of(2) * P;
                load_y();
                e2 = erows + (size_t)frame_of(3) * P;
            }
            __syncthreads();
        }
        estep = dir == 0 ? (ptrdiff_t)P : -(ptrdiff_t)P;
        tstep = dir == 0 ? (ptrdiff_t)rows : -(ptrdiff_t)rows;
        sstep = dir == 0 ? 1 : -1;
        trow = trel + (size_t)(dir == 0 ? 1 : T - 1) * rows;
        sN = scalN + (dir == 0 ? 0 : T);
        sS = scalS + (dir == 0 ? 0 : T);
        const uint32_t part_at = ((uint32_t)wave + (HAS_WB && lane >= 32 ? 16u : 0u)) * kRB;
        if (dir == 0) loop<0>(T, tid, lane, eps, aconst, bconst, mask, row4_first, ey_first, part_at, nsl);
        else loop<1>(T, tid, lane, eps, aconst, bconst, mask, row4_first, ey_first, part_at, nsl);

        // ---- last scalars and the closing dot product (the vector of step T is raw:
        // beta's in-place folding happens at the start of a step that does not come)
        {
            const uint32_t xc = (T & 1) ? kRegX1 : 0u;
            const uint32_t pc = kRegPart + ((T & 1) ? 32u * kRB : 0u);
            Real pv = lds_ldr<Real>(pc + (lane & (HAS_WB ? 31 : 15)) * kRB);
            pv = row16_allsum(pv);
            const Real N = lane_value(pv, 0);
            const Real Sd = HAS_WB ? lane_value(pv, 16) : aconst * N;
            const Real inv = N > 0 ? (Real)1 / N : (Real)0;
            const Real c = eps * Sd * inv;
            if (tid == 0) {
                const int tp = dir == 0 ? T : 0;
                scalN[tp] = N;
                scalS[tp] = Sd;
            }
            Real z = 0;
            for (int sl = s0; sl < s1; ++sl) {
                const int row = sl * 64 + lane;
                const Real v = lds_ldr<Real>(xc + row * kRB) * inv +
                               c * (Real)p.g.vb[od.vec_at + row];
                z += (Real)p.g.vfin[od.vec_at + row] * v;
            }
            z = wave_sum_uniform(z);
            __syncthreads();
            if (lane == 0) lds_st(kRegPart + (64 + wave) * kRB, z);
            __syncthreads();
            if (tid == 0) {
                Real Z = 0;
                for (int w = 0; w < (nthreads >> 6); ++w)
                    Z += lds_ldr<Real>(kRegPart + (64 + w) * kRB);
                static_cast<Real*>(p.zfin)[(size_t)dir * p.B + b] = Z;
            }
        }
    }
};

// ---------------------------------------------------------------------------
// Scales of one sequence, once both of its recursions are done:
//   log Z_b = log(zfin) + sum_t log n_t (+ the frame maxima), and the factor that
//   turns ahat_{t-1} * w * e_t * bhat_t into an occupancy,
//   c_t = exp(A_{t-1} + B_t - log Z'),  A, B = prefix / suffix sums of log n,
// in fp64. Called by every thread of a workgroup (at most 256 of them work);
// scratch: 8 KB of LDS nobody else uses.
// ---------------------------------------------------------------------------
// Largest difference (nats) between the alpha-side and the beta-side log Z of a
// sequence that counts as rounding: fp32 state vectors on the longest workloads
// here differ by a few 1e-5.
constexpr double kTotalsAgree = 1e-3;

template <typename Real>
__device__ void scan_sequence(const FbParams& p, const int b, unsigned char* scratch_raw)
{
    double* sa = reinterpret_cast<double*>(scratch_raw);
    double* sb = sa + 256;
    double* sm = sb + 256;
    double* tot = sm + 256;
    const int tid = threadIdx.x;
    const int workers = min((int)blockDim.x, 256);
    const SeqDesc sd = p.seqs[b];
    const int T = sd.T;
    const int n = T + 1;
    const Real* na = static_cast<const Real*>(p.scal) + sd.scal_at;
    const Real* nb = static_cast<const Real*>(p.scal) + 2 * p.scal_total + sd.scal_at;
    Real* cfac = static_cast<Real*>(p.cfac) + sd.scal_at;
    const int chunk = (n + workers - 1) / workers;
    const bool work = tid < workers;
    const int i0 = work ? min(tid * chunk, n) : n, i1 = min(i0 + chunk, n);
    double la = 0.0, lb = 0.0, lm = 0.0;
    for (int i = i0; i < i1; ++i) {
        la += log((double)na[i]);
        lb += log((double)nb[i]);
    }
    if (work)
        for (int t = tid; t < T; t += workers) lm += (double)p.rowmax[(size_t)b * p.T + t];
    if (work) { sa[tid] = la; sb[tid] = lb; sm[tid] = lm; }
    __syncthreads();
    if (tid == 0) {
        double ra = 0.0, rb = 0.0, rm = 0.0;
        for (int i = 0; i < workers; ++i) {
            const double xa = sa[i], xb = sb[i];
            sa[i] = ra; sb[i] = rb;  // exclusive prefixes
            ra += xa; rb += xb; rm += sm[i];
        }
        tot[0] = ra; tot[1] = rb; tot[2] = rm;
    }
    __syncthreads();
    const double totB = tot[1], msum = tot[2];
    const double lz = log((double)static_cast<const Real*>(p.zfin)[b]) + tot[0];
    // the same total from the beta side: pi . beta'_0. The two agree up to rounding
    // unless a pass lost mass to underflow (a state whose alpha is below the range
    // of Real next to the frame's total while its beta is that much above, or the
    // other way round): such a sequence is flagged, not returned silently wrong
    const double lz_beta = log((double)static_cast<const Real*>(p.zfin)[p.B + b]) + totB;
    const bool nonfinite_in = !(msum == msum);
    const bool dead = !(lz > -INFINITY && lz < INFINITY) || nonfinite_in;
    const bool lossy = !dead && !(fabs(lz - lz_beta) <= kTotalsAgree);
    double ra = work ? sa[tid] : 0.0, rb = work ? sb[tid] : 0.0;
    for (int i = i0; i < i1; ++i) {
        if (i >= 1) cfac[i] = dead ? (Real)0 : (Real)exp(ra + (totB - rb) - lz);
        ra += log((double)na[i]);
        rb += log((double)nb[i]);
    }
    if (tid == 0) {
        int st = 0;
        if (nonfinite_in) st |= 2;
        if (dead) st |= 1;
        if (lossy) st |= 4;
        const float val = nonfinite_in ? __builtin_nanf("") : (float)(lz + msum);
        const float out = p.grad_scale * val;
        p.objf[b] = p.accumulate ? p.objf[b] + out : out;
        if (p.status_out) p.status_out[b] = p.accumulate ? (p.status_out[b] | st) : st;
    }
}

template <typename Real, int NSLOT, bool YREP, bool HAS_WB, int NT, bool HYBRID = false,
          bool BIG = false, bool HUBS = false, bool GROUPED = false>
__global__ void __launch_bounds__(NT) k_rec(FbParams p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int code = p.order[2 * p.seq_first + blockIdx.x];
    const int b = code >> 1, dir = code & 1;
#ifdef LFMMI_ONLY_DIR  // timing builds only: one of the two recursions (results are not valid)
    if (dir != LFMMI_ONLY_DIR) return;
#endif
    const SeqDesc sd = p.seqs[b];
    const OrdDesc od = p.g.ords[sd.graph * 3 + dir];
    if constexpr (GROUPED) {
        static_assert(NSLOT > 0 && !YREP && !HYBRID && !BIG && !HUBS, "grouped: resident arcs only");
        RecGrouped<Real, HAS_WB, NSLOT, NT> r;
        r.run(p, sd, od, b, dir);
    } else if constexpr (NSLOT > 0) {
        RecRegs<Real, YREP, HAS_WB, NSLOT, NT, HYBRID, BIG, HUBS> r;
        r.run(p, sd, od, b, dir, lds_raw);
    } else {
        rec_run<Real, YREP, HAS_WB, NT, HUBS>(p, sd, od, b, dir, lds_raw);
    }
    // The workgroup that finishes a sequence second (alpha or beta) computes its
    // scales: no launch of their own, and no wait for the other sequences.
    __threadfence();   // this thread's trellis rows and scalars are visible device-wide
    __syncthreads();   // ... and so are everybody's; LDS is free from here on
    int* ticket = reinterpret_cast<int*>(lds_raw);
    if (threadIdx.x == 0) *ticket = atomicAdd(p.done + b, 1);
    __syncthreads();
    if (*ticket != 1) return;  // workgroup-uniform
    __threadfence();           // read the other workgroup's results from memory
    scan_sequence<Real>(p, b, lds_raw + 64);
}

// ---------------------------------------------------------------------------
// Occupancy and gradient, frames in parallel. Rows of the OCC ordering are
// pieces of one pdf's arc list; a row's sum is stored to LDS and one thread per
// pdf then adds that pdf's rows in table order, so the result does not depend
// on timing. (An LDS float atomic add takes about 190 clocks per wave
// instruction on this chip whatever its addresses, against 2 to 4 for a store.)
//   gamma_t[d] = c_t * e_t[d] * sum_{a: pdf_a = d} w_a * ahat_{t-1}[src_a] * bhat_t[dst_a]
// ---------------------------------------------------------------------------
template <typename Real>
__device__ __forceinline__ Real occ_term(const uint2 r, const Real* XA, const Real* XB)
{
    return (Real)__uint_as_float(r.y) * lds_at(XB, r.x >> 16) * lds_at(XA, r.x & 0xffffu);
}

template <typename Real>
__global__ void __launch_bounds__(1024) k_occ(FbParams p, int frames_per_wg)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x;
    const int b = p.order[2 * (p.seq_first + blockIdx.y)] >> 1;
    const SeqDesc sd = p.seqs[b];
    const int T = sd.T;
    const int P = p.P;
    const OrdDesc od = p.g.ords[sd.graph * 3 + 2];
    const int rows_f = p.g.ords[sd.graph * 3 + 0].num_slices * 64;
    const int rows_b = p.g.ords[sd.graph * 3 + 1].num_slices * 64;

    Real* XA = reinterpret_cast<Real*>(lds_raw);
    Real* XB = XA + p.lds_rows_occ_a;
    Real* rowsum = XB + p.lds_rows_occ_b;

    const uint4* recs = rec_pairs(p, od, lane);
    const int32_t* so = p.g.slice_off + od.slice_off_at;
    const int32_t* pdf_first = p.g.pdf_first + od.pdf_first_at;
    const int32_t* row_slot = p.g.row_slot + od.vec_at;
    // pdfs with more than heavy_rows rows: their row sums are added by a whole wave
    const int heavy_n = pdf_first[P + 1], heavy_rows = pdf_first[P + 2];
    const int32_t* heavy = pdf_first + P + 3;
    const Real* cfac = static_cast<const Real*>(p.cfac) + sd.scal_at;
    const Real* scal = static_cast<const Real*>(p.scal) + sd.scal_at;
    const float* vb_f = p.g.vb + p.g.ords[sd.graph * 3 + 0].vec_at;
    const float* vb_b = p.g.vb + p.g.ords[sd.graph * 3 + 1].vec_at;
    const Real eps = (Real)p.leak;
    int s0 = 0, s1 = 0;
    if (wave < od.num_waves) {
        s0 = p.g.wave_first[od.wave_first_at + wave];
        s1 = p.g.wave_first[od.wave_first_at + wave + 1];
    }

    const int t_first = blockIdx.x * frames_per_wg + 1;
    const int t_last = min(t_first + frames_per_wg - 1, p.T);
    for (int t = t_first; t <= t_last; ++t) {
        const size_t at = ((size_t)b * p.T + (t - 1)) * P;
        float* g = p.grad + at;
        const Real c = t <= T ? cfac[t] : (Real)0;
        if (t > T || c == (Real)0) {  // beyond the sequence, or a dead sequence
            if (!p.accumulate)
                for (int d = tid; d < P; d += nthreads) g[d] = 0.f;
            continue;
        }
        // the trellis holds raw vectors: vhat' = v / n + (eps * s / n) * b
        const Real na = scal[t - 1], sa = scal[p.scal_total + t - 1];
        const Real nb = scal[2 * p.scal_total + t], sb = scal[3 * p.scal_total + t];
        const Real inva = (Real)1 / na, ca = eps * sa * inva;
        const Real invb = (Real)1 / nb, cb = eps * sb * invb;
        const Real* ar = static_cast<const Real*>(p.alpha) + sd.alpha_at + (size_t)(t - 1) * rows_f;
        const Real* br = static_cast<const Real*>(p.beta) + sd.beta_at + (size_t)t * rows_b;
        for (int r = tid; r < rows_f; r += nthreads) XA[r] = ar[r] * inva + ca * (Real)vb_f[r];
        for (int r = tid; r < rows_b; r += nthreads) XB[r] = br[r] * invb + cb * (Real)vb_b[r];
        __syncthreads();
        for (int sl = s0; sl < s1; ++sl) {
            const int o0 = so[sl], o1 = so[sl + 1];
            const uint4* rp = recs + (size_t)(o0 >> 1) * 64;
            const int slot = row_slot[sl * 64 + lane];  // where this row's sum goes
            Real acc = 0;
            int i = o0;
            for (; i + 4 <= o1; i += 4) {
                const uint4 r0 = rp[0], r1 = rp[64];
                rp += 128;
                acc += occ_term(rec_lo(r0), XA, XB);
                acc += occ_term(rec_hi(r0), XA, XB);
                acc += occ_term(rec_lo(r1), XA, XB);
                acc += occ_term(rec_hi(r1), XA, XB);
            }
            for (; i < o1; i += 2) {  // widths are even
                const uint4 r0 = rp[0];
                rp += 64;
                acc += occ_term(rec_lo(r0), XA, XB);
                acc += occ_term(rec_hi(r0), XA, XB);
            }
            rowsum[slot] = acc;
        }
        __syncthreads();
        const Real scale = (Real)p.grad_scale * c;
        const float* e = p.emis + at;
        for (int d = tid; d < P; d += nthreads) {
            const int r0 = pdf_first[d], r1 = pdf_first[d + 1];
            if (r1 - r0 > heavy_rows) continue;  // a wave adds these up, below
            Real sum = 0;
            for (int r = r0; r < r1; ++r) sum += rowsum[r];
            const float v = (float)(scale * (Real)e[d] * sum);
            g[d] = p.accumulate ? g[d] + v : v;
        }
        for (int h = wave; h < heavy_n; h += nthreads >> 6) {
            const int d = heavy[h];
            Real sum = 0;
            for (int r = pdf_first[d] + lane, r1 = pdf_first[d + 1]; r < r1; r += 64)
                sum += rowsum[r];
            sum = wave_sum_uniform(sum);
            if (lane == 0) {
                const float v = (float)(scale * (Real)e[d] * sum);
                g[d] = p.accumulate ? g[d] + v : v;
            }
        }
        // the next frame's row sums are stored after its staging barrier, which
        // every thread reaches only once it is done here
    }
}

// ---------------------------------------------------------------------------
// Occupancy, F frames at a time (fp32). The arc records are the bulk of what
// the frame-at-a-time kernel pulls out of L2 (8 bytes per arc and frame), and
// every chunk of them costs an exposed L2 latency; here one record serves F
// consecutive frames. LDS holds one plane per frame and side at a fixed stride,
//   XA[f] at f * STRIDE, XB[f] at (F + f) * STRIDE, row sums [f][row] after them,
// so a gather is a 4-byte read at the record's state offset plus an immediate,
// with the bank pattern the packer ordered the slots for. Thread f * P + d then
// adds the row sums of pdf d in frame f and writes that gradient entry: the F
// gradient rows of a group are contiguous, so the write is coalesced.
// ---------------------------------------------------------------------------
template <int F, int STRIDE>
__global__ void __launch_bounds__(1024) k_occ_planes(FbParams p, int groups_per_wg)
{
    LFMMI_MARK_BEGIN
    // Plane offsets ride in the 16-bit immediate of the ds instruction. Where the XB
    // planes lie beyond 64 KB (two frames of 32 KB planes), the record's XB offset is
    // taken out of its upper half together with a 1 above it (64 KB + offset, one
    // instruction as the shift would be) and the immediate holds the rest.
    constexpr bool kBHigh = (2 * F - 1) * STRIDE > 65535;
    static_assert((F - 1) * STRIDE <= 65535, "XA plane offsets must fit the ds immediate");
    static_assert(!kBHigh || (F * STRIDE >= 65536 && (2 * F - 1) * STRIDE - 65536 <= 65535),
                  "XB plane offsets less 64 KB must fit the ds immediate");
    constexpr uint32_t kBBase = kBHigh ? 65536u : 0u;
    constexpr uint32_t kRowSum = 2u * F * STRIDE;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x;
    const int b = p.order[2 * (p.seq_first + blockIdx.y)] >> 1;
    const SeqDesc sd = p.seqs[b];
    const int T = sd.T;
    const int P = p.P;
    const OrdDesc od = p.g.ords[sd.graph * 3 + 2];
    const OrdDesc odf = p.g.ords[sd.graph * 3 + 0];
    const OrdDesc odb = p.g.ords[sd.graph * 3 + 1];
    const int rows_f = odf.num_slices * 64, rows_b = odb.num_slices * 64;
    const int occ_rows = od.num_slices * 64;

    const uint4* recs = rec_pairs(p, od, lane);
    const int32_t* so = p.g.slice_off + od.slice_off_at;
    const int32_t* pdf_first = p.g.pdf_first + od.pdf_first_at;
    const int32_t* row_slot = p.g.row_slot + od.vec_at;
    const int heavy_n = pdf_first[P + 1], heavy_rows = pdf_first[P + 2];
    const int32_t* heavy = pdf_first + P + 3;
    const float* scal = static_cast<const float*>(p.scal) + sd.scal_at;
    const float* cfac = static_cast<const float*>(p.cfac) + sd.scal_at;
    const float* vb_f = p.g.vb + odf.vec_at;
    const float* vb_b = p.g.vb + odb.vec_at;
    const float* alpha = static_cast<const float*>(p.alpha) + sd.alpha_at;
    const float* beta = static_cast<const float*>(p.beta) + sd.beta_at;
    const float eps = p.leak;
    int s0 = 0, s1 = 0;
    if (wave < od.num_waves) {
        s0 = p.g.wave_first[od.wave_first_at + wave];
        s1 = p.g.wave_first[od.wave_first_at + wave + 1];
    }
    // this thread's first gradient entry of a group: frame my_f, pdf my_d, whose row
    // sums are the words my_r0 .. my_r1 - 1 of a frame's row sums
    const int my_f = tid / P, my_d = tid - my_f * P;
    int my_r0 = 0, my_r1 = 0;
    if (my_f < F) {
        my_r0 = pdf_first[my_d];
        my_r1 = pdf_first[my_d + 1];
    }
    // one frame per group: a thread writes the same pdfs tid + j * nthreads in every
    // frame; the row ranges of the next kMore of them stay in registers too
    constexpr int kMore = F == 1 ? 2 : 0;
    int more_r0[kMore ? kMore : 1], more_r1[kMore ? kMore : 1];
#pragma unroll
    for (int j = 0; j < kMore; ++j) {
        const int d = tid + (j + 1) * nthreads;
        more_r0[j] = d < P ? pdf_first[d] : 0;
        more_r1[j] = d < P ? pdf_first[d + 1] : 0;
    }
    // pdfs with many rows: wave w adds up (pdf, frame) pairs w, w + nwaves, ... of every
    // group; the row ranges of its first kHeavyKept pairs stay in registers
    constexpr int kHeavyKept = 2;
    const int nwaves = nthreads >> 6;
    int hv_d[kHeavyKept], hv_r0[kHeavyKept], hv_r1[kHeavyKept];
#pragma unroll
    for (int k = 0; k < kHeavyKept; ++k) {
        const int u = wave + k * nwaves;
        hv_d[k] = hv_r0[k] = hv_r1[k] = 0;
        if (u < heavy_n * F) {
            hv_d[k] = heavy[u / F];
            hv_r0[k] = pdf_first[hv_d[k]];
            hv_r1[k] = pdf_first[hv_d[k] + 1];
        }
    }
    // Where the sums of this lane's rows go among the row sums (a pdf's rows side by
    // side), one place per slice of the wave: the variants with large planes (one
    // workgroup per compute unit whatever they add to their LDS) keep the table behind
    // the row sums, the others keep the wave's first kSlotsKept slices in registers
    // and fetch the place of a later slice when it ends.
    // lane l: one past the last slot of the wave's l-th slice (its last slice's from there
    // on); the wave's first slot and one past its last
    const int so_tab = s0 < s1 ? so[min(s0 + 1 + lane, s1)] : 0;
    const int w0 = s0 < s1 ? so[s0] : 0, w1 = s0 < s1 ? so[s1] : 0;
    constexpr bool kSlotsInLds = STRIDE >= 32768;
    constexpr int kSlotsKept = kSlotsInLds ? 1 : 4;
    const uint32_t slot_tab = kRowSum + (uint32_t)(F * occ_rows) * 4u;
    uint32_t slot_r[kSlotsKept];
    if constexpr (kSlotsInLds) {
        slot_r[0] = 0;
        for (int sl = s0; sl < s1; ++sl)  // read back by this wave only
            lds_st(slot_tab + (uint32_t)(sl * 64 + lane) * 4u,
                   __uint_as_float((uint32_t)row_slot[sl * 64 + lane]));
    } else {
#pragma unroll
        for (int q = 0; q < kSlotsKept; ++q)
            slot_r[q] = s0 < s1 ? (uint32_t)row_slot[min(s0 + q, s1 - 1) * 64 + lane] : 0u;
    }
    // ... and the rows of the next group are fetched while this group's arcs are
    // gathered: kStageRows of each side and frame per thread (large planes, where one
    // workgroup has a compute unit to itself; uniform leak target only)
    constexpr bool kAhead = F == 1 || (F == 2 && STRIDE == 32768);
    constexpr int kStageRows = kAhead ? STRIDE / 4096 : 1;
    const int rows_most = max(rows_f, rows_b);
    const bool ahead = kAhead && !odf.has_wb && nthreads * kStageRows >= rows_most;
    float next_a[kAhead ? F : 1][kStageRows], next_b[kAhead ? F : 1][kStageRows];
    // alpha of frames t - 1 .., beta of frames t .., as stored (zeros past the sequence)
    auto fetch_rows = [&](const int t) {
#pragma unroll
        for (int f = 0; f < (kAhead ? F : 1); ++f) {
            const bool live = t + f <= T;
#pragma unroll
            for (int u = 0; u < kStageRows; ++u) {
                int r = u * nthreads + tid;
                asm volatile("" : "+v"(r));  // recomputed here: no address registers held per row
                next_a[f][u] = (live && r < rows_f) ? alpha[(size_t)(t + f - 1) * rows_f + r] : 0.f;
                next_b[f][u] = (live && r < rows_b) ? beta[(size_t)(t + f) * rows_b + r] : 0.f;
            }
        }
    };

    const int t_begin = blockIdx.x * groups_per_wg * F + 1;
    const int t_end = min(t_begin + groups_per_wg * F - 1, p.T);
    if constexpr (kAhead)
        if (ahead && t_begin <= min(t_end, T)) fetch_rows(t_begin);
    LFMMI_MARK(0)  // start of the workgroup: descriptors, tables
    LFMMI_COUNT(14)
    for (int t0 = t_begin; t0 <= t_end; t0 += F) {
        if (t0 > T) {  // nothing but padding rows from here on
            if (!p.accumulate)
                for (int t = t0; t <= t_end; ++t) {
                    float* g = p.grad + ((size_t)b * p.T + (t - 1)) * P;
                    for (int d = tid; d < P; d += nthreads) g[d] = 0.f;
                }
            break;
        }
        // per-frame scalars: the trellis holds raw vectors, vhat' = v / n + (eps s / n) b
        float inva[F], ca[F], invb[F], cb[F], cf[F];
#pragma unroll
        for (int f = 0; f < F; ++f) {
            const int t = t0 + f;
            const bool live = t <= T;
            cf[f] = live ? cfac[t] : 0.f;
            const float na = live ? scal[t - 1] : 1.f, sa = live ? scal[p.scal_total + t - 1] : 0.f;
            const float nb = live ? scal[2 * p.scal_total + t] : 1.f;
            const float sb = live ? scal[3 * p.scal_total + t] : 0.f;
            const bool ok = live && cf[f] != 0.f;  // dead sequences stage zeros
            inva[f] = ok ? 1.f / na : 0.f;
            ca[f] = eps * sa * inva[f];
            invb[f] = ok ? 1.f / nb : 0.f;
            cb[f] = eps * sb * invb[f];
        }
        LFMMI_MARK(1)  // the group's scales
        __syncthreads();  // the previous group's gathers and row-sum reads are done
        LFMMI_MARK(2)
        // staging: two rows per thread and side in flight, all loads (alpha and beta)
        // issued before any is used
        const int rows_max = ahead ? 0 : rows_most;
        if constexpr (kAhead)
            if (ahead) {
#pragma unroll
                for (int f = 0; f < F; ++f) {
                    const float la = ca[f] * odf.b_const, lb = cb[f] * odb.b_const;
#pragma unroll
                    for (int u = 0; u < kStageRows; ++u) {
                        int r = u * nthreads + tid;
                        asm volatile("" : "+v"(r));
                        if (r < rows_f)
                            lds_st((uint32_t)(f * STRIDE) + (uint32_t)r * 4u,
                                   fmaf(next_a[f][u], inva[f], la));
                        if (r < rows_b)
                            lds_st((uint32_t)((F + f) * STRIDE) + (uint32_t)r * 4u,
                                   fmaf(next_b[f][u], invb[f], lb));
                    }
                }
            }
        for (int r0 = 0; r0 < rows_max; r0 += 2 * nthreads) {
            float va[2][F], vbt[2][F], ba[2], bbt[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = r0 + u * nthreads + tid;
                ba[u] = r < rows_f ? vb_f[r] : 0.f;
                bbt[u] = r < rows_b ? vb_b[r] : 0.f;
#pragma unroll
                for (int f = 0; f < F; ++f) {
                    const bool live = t0 + f <= T;
                    va[u][f] = (r < rows_f && live) ? alpha[(size_t)(t0 - 1 + f) * rows_f + r] : 0.f;
                    vbt[u][f] = (r < rows_b && live) ? beta[(size_t)(t0 + f) * rows_b + r] : 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = r0 + u * nthreads + tid;
#pragma unroll
                for (int f = 0; f < F; ++f) {
                    if (r < rows_f)
                        lds_st((uint32_t)(f * STRIDE) + (uint32_t)r * 4u,
                               fmaf(va[u][f], inva[f], ca[f] * ba[u]));
                    if (r < rows_b)
                        lds_st((uint32_t)((F + f) * STRIDE) + (uint32_t)r * 4u,
                               fmaf(vbt[u][f], invb[f], cb[f] * bbt[u]));
                }
            }
        }
        LFMMI_MARK(3)  // staging
        __syncthreads();
        LFMMI_MARK(4)
        if constexpr (kAhead)
            if (ahead && t0 + F <= min(t_end, T)) fetch_rows(t0 + F);

        // emission value and frame scale of this thread's gradient entry, in flight
        // during the gathers
        const size_t group_at = ((size_t)b * p.T + (t0 - 1)) * P;
        const bool my_live = my_f < F && t0 + my_f <= T;
        const float my_e = my_live ? p.emis[group_at + tid] : 0.f;
        const float my_c = my_live ? cfac[t0 + my_f] : 0.f;
        float more_e[kMore ? kMore : 1];
#pragma unroll
        for (int j = 0; j < kMore; ++j) {
            const int d = tid + (j + 1) * nthreads;
            more_e[j] = d < P ? p.emis[group_at + d] : 0.f;
        }
        // ... and those of the (pdf, frame) pairs this wave adds up with all its lanes
        float hv_e[kHeavyKept], hv_c[kHeavyKept];
#pragma unroll
        for (int k = 0; k < kHeavyKept; ++k) {
            const int u = wave + k * nwaves;
            const int f = u % F;
            const bool on = u < heavy_n * F && t0 + f <= T;
            hv_e[k] = on ? p.emis[group_at + (size_t)f * P + hv_d[k]] : 0.f;
            hv_c[k] = on ? cfac[t0 + f] : 0.f;
        }

        if (s0 < s1) {
            // The wave's slices as one flat sequence of record pairs (slices are an even
            // number of slots wide, so a pair never straddles two): kChunk pairs are being
            // used while the kChunk after them load, across slice ends, so that a slice
            // does not start with an exposed trip to L2. A load past the wave's last pair
            // fetches that pair again, unused (a conditional 16-byte load would be split
            // into four 4-byte ones). The gathers of kBatch slots (16 reads) go out
            // together and are waited for once; left to itself the compiler waits for
            // every slot's reads before it issues the next slot's. Where a slice ends,
            // the lane's sums go to its row's place among the row sums. Everything that
            // steers the loop is wave-uniform and sits in scalar registers.
            constexpr int kChunk = 4;
            constexpr int kBatch = 8 / F;  // slots per batch of gathers
            static_assert((2 * kChunk) % kBatch == 0, "a chunk is a whole number of batches");
            // (the end of the wave's k-th slice: out of a lane of so_tab, no memory access)
            auto slice_end = [&](const int k) {
                return k < 64 ? __builtin_amdgcn_readlane(so_tab, __builtin_amdgcn_readfirstlane(k))
                              : so[min(s0 + k + 1, s1)];
            };
            const int q_last = (w1 >> 1) - 1;
            int sl = s0;
            int o_end = slice_end(0);
            float acc[F];
#pragma unroll
            for (int f = 0; f < F; ++f) acc[f] = 0.f;
            uint4 cur[kChunk], nxt[kChunk];
#pragma unroll
            for (int u = 0; u < kChunk; ++u) cur[u] = recs[(size_t)min((w0 >> 1) + u, q_last) * 64];
            for (int i = w0; i < w1; i += 2 * kChunk) {
#pragma unroll
                for (int u = 0; u < kChunk; ++u)
                    nxt[u] = recs[(size_t)min((i >> 1) + kChunk + u, q_last) * 64];
#pragma unroll
                for (int v0 = 0; v0 < 2 * kChunk; v0 += kBatch) {  // v: slot of the chunk
                    if (i + v0 >= w1) break;
                    // (pairs past the wave's end repeat its last pair: reads in bounds, unused)
                    float va[kBatch][F], vb[kBatch][F], w[kBatch];
#pragma unroll
                    for (int v = 0; v < kBatch; ++v) {
                        const uint4 pr = cur[(v0 + v) >> 1];
                        const uint2 r = ((v0 + v) & 1) ? rec_hi(pr) : rec_lo(pr);
                        const uint32_t xa = r.x & 0xffffu;
                        const uint32_t xb = kBHigh ? __builtin_amdgcn_alignbit(1u, r.x, 16u) : r.x >> 16;
                        w[v] = __uint_as_float(r.y);
#pragma unroll
                        for (int f = 0; f < F; ++f) {
                            va[v][f] = lds_ld(xa + (uint32_t)(f * STRIDE));
                            vb[v][f] = lds_ld(xb + ((uint32_t)((F + f) * STRIDE) - kBBase));
                        }
                    }
                    {  // one wait for the batch: the values used first depend on all the others
                        float* a = &va[0][0];
                        float* b = &vb[0][0];
#pragma unroll
                        for (int j = 1; j < kBatch * F; ++j)
                            asm volatile("" : "+v"(a[0]), "+v"(b[0]) : "v"(a[j]), "v"(b[j]));
                    }
#pragma unroll
                    for (int v = 0; v < kBatch; ++v) {
                        const int at = i + v0 + v;  // this slot
                        if (v > 0 && at >= w1) break;
#pragma unroll
                        for (int f = 0; f < F; ++f) acc[f] = fmaf(w[v] * vb[v][f], va[v][f], acc[f]);
                        if (((v0 + v) & 1) && at + 1 == o_end) {  // the slice ends with this pair
                            const int k = sl - s0;
                            uint32_t slot;
                            if constexpr (kSlotsInLds) {
                                slot = __float_as_uint(lds_ld(slot_tab + (uint32_t)(sl * 64 + lane) * 4u));
                            } else {
                                slot = slot_r[0];
#pragma unroll
                                for (int q = 1; q < kSlotsKept; ++q)
                                    if (q == k) slot = slot_r[q];
                                if (k >= kSlotsKept) slot = (uint32_t)row_slot[sl * 64 + lane];
                            }
#pragma unroll
                            for (int f = 0; f < F; ++f) {
                                lds_st(kRowSum + ((uint32_t)(f * occ_rows) + slot) * 4u, acc[f]);
                                acc[f] = 0.f;
                            }
                            ++sl;
                            o_end = slice_end(sl - s0);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kChunk; ++u) cur[u] = nxt[u];
            }
        }
        LFMMI_MARK(5)  // gathers
        __syncthreads();
        LFMMI_MARK(6)
        LFMMI_COUNT(15)
        // a pdf's row sums lie side by side; a thread adds up those of a pdf with few rows
        auto few_rows = [&](const int f, const int r0, const int r1) {
            const uint32_t at = kRowSum + (uint32_t)(f * occ_rows + r0) * 4u;
            const int cnt = r1 - r0;
            float sum = 0.f;
            // eight reads in flight at once: past the end the last word again, unused
            for (int k0 = 0; k0 < cnt; k0 += 8) {
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    v[k] = lds_ld(at + (uint32_t)min(k0 + k, cnt - 1) * 4u);
#pragma unroll
                for (int k = 0; k < 8; ++k) sum += k0 + k < cnt ? v[k] : 0.f;
            }
            return sum;
        };
        if constexpr (kMore > 0) {  // F == 1: frame t0 <= T, pdf = idx
#pragma unroll
            for (int j = 0; j < kMore; ++j) {
                const int d = tid + (j + 1) * nthreads;
                if (d >= P || more_r1[j] - more_r0[j] > heavy_rows) continue;
                const float sum = few_rows(0, more_r0[j], more_r1[j]);
                float* g = p.grad + group_at + d;
                const float v = my_c == 0.f ? 0.f : p.grad_scale * my_c * more_e[j] * sum;
                *g = p.accumulate ? *g + v : v;
            }
        }
        for (int idx = tid; idx < F * P; idx += nthreads) {
            if (kMore > 0 && idx > tid && idx <= tid + kMore * nthreads) continue;  // done above
            const int f = idx / P, d = idx - f * P;
            const int t = t0 + f;
            if (t > p.T) break;
            float* g = p.grad + group_at + idx;
            if (t > T) {
                if (!p.accumulate) *g = 0.f;
                continue;
            }
            float e, c;
            int r0, r1;
            if (idx == tid) {
                r0 = my_r0;
                r1 = my_r1;
                e = my_e;
                c = my_c;
            } else {
                r0 = pdf_first[d];
                r1 = pdf_first[d + 1];
                e = p.emis[group_at + idx];
                c = cfac[t];
            }
            if (r1 - r0 > heavy_rows) continue;  // a wave adds these up, below
            const float sum = few_rows(f, r0, r1);
            const float v = c == 0.f ? 0.f : p.grad_scale * c * e * sum;
            *g = p.accumulate ? *g + v : v;
        }
        LFMMI_MARK(7)  // sums of the pdfs with few rows
        // pdfs with many rows: one wave per pdf and frame, lanes striding over the rows
        for (int u = wave, k = 0; u < heavy_n * F; u += nwaves, ++k) {
            const int h = u / F, f = u - h * F;
            const int t = t0 + f;
            if (t > T) continue;  // zeroed above
            int d = 0, r0 = 0, r1 = 0;
            float e = 0.f, c = 0.f;
            if (k < kHeavyKept) {
#pragma unroll
                for (int q = 0; q < kHeavyKept; ++q)
                    if (q == k) {
                        d = hv_d[q];
                        r0 = hv_r0[q];
                        r1 = hv_r1[q];
                        e = hv_e[q];
                        c = hv_c[q];
                    }
            } else {
                d = heavy[h];
                r0 = pdf_first[d];
                r1 = pdf_first[d + 1];
                e = p.emis[group_at + (size_t)f * P + d];
                c = cfac[t];
            }
            float sum = 0.f;
            for (int r = r0 + lane; r < r1; r += 64)
                sum += lds_ld(kRowSum + (uint32_t)(f * occ_rows + r) * 4u);
            sum = wave_sum_uniform(sum);
            if (lane == 0) {
                float* g = p.grad + group_at + (size_t)f * P + d;
                const float v = c == 0.f ? 0.f : p.grad_scale * c * e * sum;
                *g = p.accumulate ? *g + v : v;
            }
        }
        LFMMI_MARK(8)  // sums of the pdfs with many rows
    }
}

// ---- kernel variants ---------------------------------------------------------
using RecKernel = void (*)(FbParams);
constexpr int kHybridSlots = 36;

struct RecVariant {
    int wide, nslot, yrep, has_wb, max_threads;
    RecKernel fn;
    int hybrid = 0;  // 1: hybrid, 2: hybrid with the large LDS map
    int hubs = 0;    // handles hub slices
    int grouped = 0; // emission by entered state: no emission gather (RecGrouped)
};
#define LFMMI_REC_GROUPED(REAL, WIDE, NSLOT, WB, NT)                                             \
    {WIDE, NSLOT, 0, WB, NT, k_rec<REAL, NSLOT, false, (WB != 0), NT, false, false, false, true>, \
     0, 0, 1}

#define LFMMI_REC(REAL, WIDE, NSLOT, WB, NT)                                                    \
    {WIDE, NSLOT, 0, WB, NT, k_rec<REAL, NSLOT, false, (WB != 0), NT>},                         \
    {WIDE, NSLOT, 1, WB, NT, k_rec<REAL, NSLOT, true, (WB != 0), NT>},                          \
    {WIDE, NSLOT, 0, WB, NT, k_rec<REAL, NSLOT, false, (WB != 0), NT, false, false, true>, 0, 1}, \
    {WIDE, NSLOT, 1, WB, NT, k_rec<REAL, NSLOT, true, (WB != 0), NT, false, false, true>, 0, 1}
const RecVariant kRecVariants[] = {
    // streamed arcs
    LFMMI_REC(float, 0, 0, 0, 1024), LFMMI_REC(float, 0, 0, 1, 1024),
    LFMMI_REC(double, 1, 0, 0, 1024), LFMMI_REC(double, 1, 0, 1, 1024),
    // register-resident arcs, 16 waves (128 VGPRs per lane)
    LFMMI_REC(float, 0, 16, 0, 1024), LFMMI_REC(float, 0, 20, 0, 1024),
    LFMMI_REC(float, 0, 24, 0, 1024), LFMMI_REC(float, 0, 26, 0, 1024),
    // (28 slots with hub code and a replicated emission row would spill a register)
    {0, 28, 0, 0, 1024, k_rec<float, 28, false, false, 1024>},
    {0, 28, 1, 0, 1024, k_rec<float, 28, true, false, 1024>},
    {0, 28, 0, 0, 1024, k_rec<float, 28, false, false, 1024, false, false, true>, 0, 1},
    LFMMI_REC(float, 0, 16, 1, 1024),
    // register-resident arcs, 12 waves (168 VGPRs per lane)
    LFMMI_REC(float, 0, 32, 0, 768), LFMMI_REC(float, 0, 36, 0, 768),
    // register-resident arcs, 8 waves (256 VGPRs per lane)
    LFMMI_REC(float, 0, 32, 0, 512), LFMMI_REC(float, 0, 48, 0, 512),
    LFMMI_REC(float, 0, 32, 1, 512),
    // (48 slots with per-arc leak factors: plain emission rows only, no spill)
    {0, 48, 0, 1, 512, k_rec<float, 48, false, true, 512>},
    {0, 48, 0, 1, 512, k_rec<float, 48, false, true, 512, false, false, true>, 0, 1},
    // fp64 state vectors (graphs with non-final states: numerators are small)
    LFMMI_REC(double, 1, 8, 1, 1024), LFMMI_REC(double, 1, 16, 1, 1024),
    LFMMI_REC(double, 1, 32, 1, 512),
    LFMMI_REC(double, 1, 16, 0, 1024), LFMMI_REC(double, 1, 32, 0, 512),
    // hybrid: kHybridSlots slots of a wave in registers, its other slices streamed
    {0, kHybridSlots, 0, 0, 1024, k_rec<float, kHybridSlots, false, false, 1024, true>, 1},
    {0, kHybridSlots, 1, 0, 1024, k_rec<float, kHybridSlots, true, false, 1024, true>, 1},
    // ... with the LDS map for up to 12288 states
    {0, kHybridSlots, 0, 0, 1024, k_rec<float, kHybridSlots, false, false, 1024, true, true>, 2},
    // ... and the three for graphs with hub slices
    // (with a replicated emission row the hub code would spill a register: plain rows)
    {0, kHybridSlots, 0, 0, 1024, k_rec<float, kHybridSlots, false, false, 1024, true, false, true>, 1, 1},
    {0, kHybridSlots, 0, 0, 1024, k_rec<float, kHybridSlots, false, false, 1024, true, true, true>, 2, 1},
    // emission by entered state (two registers per slot: more slots fit)
    LFMMI_REC_GROUPED(float, 0, 16, 0, 1024), LFMMI_REC_GROUPED(float, 0, 24, 0, 1024),
    LFMMI_REC_GROUPED(float, 0, 32, 0, 1024), LFMMI_REC_GROUPED(float, 0, 48, 0, 512),
    LFMMI_REC_GROUPED(float, 0, 16, 1, 1024), LFMMI_REC_GROUPED(float, 0, 24, 1, 1024),
    LFMMI_REC_GROUPED(double, 1, 8, 1, 1024), LFMMI_REC_GROUPED(double, 1, 16, 1, 512),
    LFMMI_REC_GROUPED(double, 1, 16, 0, 1024),
};
#undef LFMMI_REC
#undef LFMMI_REC_GROUPED

const RecVariant* find_rec(bool wide, int nslot, bool yrep, bool has_wb, int hybrid, bool hubs,
                           bool grouped)
{
    for (const RecVariant& v : kRecVariants)
        if (v.wide == (wide ? 1 : 0) && v.nslot == nslot && v.has_wb == (has_wb ? 1 : 0) &&
            v.grouped == (grouped ? 1 : 0) &&
            (grouped || (v.yrep == (yrep ? 1 : 0) && v.hybrid == hybrid && v.hubs == (hubs ? 1 : 0))))
            return &v;
    return nullptr;
}

}  // namespace

int rec_register_slots(bool wide, bool has_wb, bool yrep, bool hubs, int max_wave_slots,
                       int threads)
{
    int best = 0;
    for (const RecVariant& v : kRecVariants)
        if (v.wide == (wide ? 1 : 0) && v.has_wb == (has_wb ? 1 : 0) && v.nslot > 0 && !v.hybrid &&
            !v.grouped && v.yrep == (yrep ? 1 : 0) && v.hubs == (hubs ? 1 : 0) &&
            v.nslot >= max_wave_slots && threads <= v.max_threads && (best == 0 || v.nslot < best))
            best = v.nslot;
    return best;
}

int rec_grouped_slots(bool wide, bool has_wb, int max_wave_slots, int threads)
{
    int best = 0;
    for (const RecVariant& v : kRecVariants)
        if (v.grouped && v.wide == (wide ? 1 : 0) && v.has_wb == (has_wb ? 1 : 0) &&
            v.nslot >= max_wave_slots && threads <= v.max_threads && (best == 0 || v.nslot < best))
            best = v.nslot;
    return best;
}

int rec_grouped_max_rows(int threads) { return kGroupedPasses * threads; }

int rec_hybrid_slots(bool wide, bool has_wb, bool yrep, bool hubs, int map)
{
    for (const RecVariant& v : kRecVariants)
        if (v.hybrid == map && v.wide == (wide ? 1 : 0) && v.has_wb == (has_wb ? 1 : 0) &&
            v.yrep == (yrep ? 1 : 0) && v.hubs == (hubs ? 1 : 0))
            return v.nslot;
    return 0;
}

hipError_t configure_kernels()
{
    // Kernels that address LDS by absolute offsets take the dynamic allocation to
    // start at 0: a static allocation (say a private array the compiler moved to
    // LDS) would sit there instead and be overwritten.
    auto no_static_lds = [](const void* f) {
        hipFuncAttributes attr;
        const hipError_t e = hipFuncGetAttributes(&attr, f);
        if (e != hipSuccess) return e;
        return attr.sharedSizeBytes == 0 ? hipSuccess : hipErrorInvalidConfiguration;
    };
    for (const RecVariant& v : kRecVariants) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(v.fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        if (v.nslot > 0 && (e = no_static_lds(reinterpret_cast<const void*>(v.fn))) != hipSuccess)
            return e;
    }
    const void* fns[] = {reinterpret_cast<const void*>(k_occ<float>),
                         reinterpret_cast<const void*>(k_occ<double>),
                         reinterpret_cast<const void*>(k_occ_planes<4, 8192>),
                         reinterpret_cast<const void*>(k_occ_planes<2, 16384>),
                         reinterpret_cast<const void*>(k_occ_planes<2, 32768>),
                         reinterpret_cast<const void*>(k_occ_planes<1, 32768>),
                         reinterpret_cast<const void*>(k_occ_planes<1, 49152>)};
    for (const void* f : fns) {
        hipError_t e =
            hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        if (f != fns[0] && f != fns[1] && (e = no_static_lds(f)) != hipSuccess) return e;
    }
    return hipSuccess;
}

size_t rec_lds_bytes(int lds_rows, int P, bool wide, bool yrep)
{
    const size_t ylen = yrep ? (size_t)P * 32 : (size_t)P;
    const size_t ypad = (ylen + 63) & ~(size_t)63;
    return (2 * (size_t)lds_rows + 64) * (wide ? 8 : 4) + 2 * ypad * 4;
}

size_t occ_lds_bytes(int rows_a, int rows_b, int occ_rows, bool wide)
{
    return ((size_t)rows_a + rows_b + occ_rows) * (wide ? 8 : 4);
}

// Bytes between the planes of the plane-layout occupancy kernel for this many
// state rows and frames per record (one frame: a wider plane for large graphs).
static int occ_plane_stride(int rows, int frames)
{
    if (frames == 1) return rows * 4 > 32768 ? 49152 : 32768;
    if (frames == 2) return rows * 4 > 16384 ? 32768 : 16384;
    return 8192;
}

// Frames per record of the plane-layout occupancy kernel for this many state
// rows and OCC rows (0: they do not fit its LDS map).
int occ_plane_frames(int rows, int occ_rows, int most)
{
    for (int f : {4, 2, 1})
        if (f <= most && rows * 4 <= (f == 1 ? 49152 : (f == 2 ? 32768 : 8192)) &&
            occ_plane_lds_bytes(rows, occ_rows, f) <= 160 * 1024)
            return f;
    return 0;
}

size_t occ_plane_lds_bytes(int rows, int occ_rows, int frames)
{
    // planes, row sums, and behind them (large planes only) the table of the rows' places
    const int stride = occ_plane_stride(rows, frames);
    return 2 * (size_t)frames * stride + (size_t)frames * occ_rows * 4 +
           (stride >= 32768 ? (size_t)occ_rows * 4 : 0);
}

template <typename Real>
static hipError_t launch_typed(const FbParams& p, const LaunchShape& shape, hipStream_t stream,
                               hipEvent_t* ev, const Buckets& bk)
{
    hipError_t e;
    const bool wide = sizeof(Real) == 8;
    const RecVariant* rv =
        find_rec(wide, shape.rec_nslot, shape.rec_yrep != 0, shape.rec_has_wb != 0,
                 shape.rec_hybrid, shape.rec_hubs != 0, shape.rec_grouped != 0);
    if (!rv || shape.rec_threads > rv->max_threads) return hipErrorInvalidConfiguration;
    if (bk.n > 1 && (e = hipEventRecord(bk.fork, stream)) != hipSuccess) return e;

    int rec_threads = shape.rec_threads;
    if (shape.rec_nslot > 0 && !shape.rec_grouped) {
        // enough threads to stage one emission row in the variant's passes; waves
        // beyond the graph's own hold no arcs
        const int units = shape.rec_yrep ? p.P * 8 : p.P;
        const int passes = stage_passes(shape.rec_yrep != 0, rv->max_threads);
        const int need = ((units + passes - 1) / passes + 63) / 64 * 64;
        rec_threads = std::max(rec_threads, need);
        if (rec_threads > rv->max_threads) return hipErrorInvalidConfiguration;
    }
    // at least the scan's scratch
    const size_t rec_lds =
        std::max<size_t>(shape.rec_nslot > 0
                             ? reg_lds_bytes()
                             : rec_lds_bytes(p.lds_rows, p.P, wide, shape.rec_yrep != 0),
                         8192 + 64);
    // bucket 0 (the longest sequences) first, on the caller's stream
    for (int q = 0; q < bk.n; ++q) {
        if (bk.count[q] <= 0) continue;
        hipStream_t on = q == 0 ? stream : bk.streams[q];
        if (q > 0 && (e = hipStreamWaitEvent(on, bk.fork, 0)) != hipSuccess) return e;
        FbParams pq = p;
        pq.seq_first = bk.first[q];
        const int nb = bk.count[q];
        hipEvent_t* evq = ev ? ev + 4 * q : nullptr;
#define LFMMI_EVQ(i) \
    if (evq && (!shape.profile_rec_only || i == 1 || i == 2)) { \
        e = hipEventRecord(evq[i], on); \
        if (e != hipSuccess) return e; \
    }
        LFMMI_EVQ(0)
        {  // also when T == 0: it resets the per-sequence tickets of k_rec
            dim3 grid(std::max(1, (p.T + 3) / 4), nb);
            hipLaunchKernelGGL(k_emit, grid, dim3(256), 0, on, pq);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        LFMMI_EVQ(1)
        hipLaunchKernelGGL(rv->fn, dim3(2 * nb), dim3(rec_threads), rec_lds, on, pq);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        LFMMI_EVQ(2)
        const int tq = std::min(bk.tmax[q], p.T);
        if (tq > 0) {
            if (!wide && shape.occ_multi > 0) {
                const int F = shape.occ_multi;
                const int per_wg = F * shape.occ_groups;
                dim3 grid((tq + per_wg - 1) / per_wg, nb);
                void (*fn)(FbParams, int) =
                    F == 4   ? k_occ_planes<4, 8192>
                    : F == 2 ? (occ_plane_stride(p.lds_rows, 2) == 16384 ? k_occ_planes<2, 16384>
                                                                         : k_occ_planes<2, 32768>)
                    : occ_plane_stride(p.lds_rows, 1) == 32768 ? k_occ_planes<1, 32768>
                                                               : k_occ_planes<1, 49152>;
                hipLaunchKernelGGL(fn, grid, dim3(shape.occ_threads),
                                   occ_plane_lds_bytes(p.lds_rows, p.lds_rows_occ, F), on, pq,
                                   shape.occ_groups);
            } else {
                dim3 grid((tq + shape.occ_frames - 1) / shape.occ_frames, nb);
                hipLaunchKernelGGL(k_occ<Real>, grid, dim3(shape.occ_threads),
                                   occ_lds_bytes(p.lds_rows_occ_a, p.lds_rows_occ_b,
                                                 p.lds_rows_occ, wide),
                                   on, pq, shape.occ_frames);
            }
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        LFMMI_EVQ(3)
#undef LFMMI_EVQ
    }
    // Join: the streams wait for one another in a chain, last bucket first, and the
    // caller's stream for the head of the chain only. Its own bucket ends last as a
    // rule, and every wait it has to process then delays whatever follows the call.
    int after = -1;  // the stream whose join event the next one in the chain waits for
    for (int q = bk.n - 1; q >= 1; --q) {
        if (bk.count[q] <= 0) continue;
        if (after > 0 && (e = hipStreamWaitEvent(bk.streams[q], bk.join[after], 0)) != hipSuccess)
            return e;
        if ((e = hipEventRecord(bk.join[q], bk.streams[q])) != hipSuccess) return e;
        after = q;
    }
    if (after > 0 && (e = hipStreamWaitEvent(stream, bk.join[after], 0)) != hipSuccess) return e;
    return hipSuccess;
}

// ---- the allocation-free entry point's workspace --------------------------------
// For callers that cannot allocate (HIP graph capture, serving loops): the
// workspace of a call sits in this array instead of in memory the handle
// allocates. Each GPU the library runs on holds its own copy, at its own address,
// until the process ends; the array's name is only a host-side stand-in, so host
// code uses the address hipGetSymbolAddress returned for the device.
namespace {
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

struct StaticLengths {
    int32_t T[kStaticMaxBatch];
};

// One workgroup: what the host writes for the allocating entry point, computed
// here. Sequences are launched longest first (by frames times arc slots).
__global__ void __launch_bounds__(kStaticMaxBatch) k_describe(FbParams p, StaticLengths len,
                                                              int num_graphs)
{
    __shared__ long long work[kStaticMaxBatch];
    SeqDesc* seqs = const_cast<SeqDesc*>(p.seqs);
    int32_t* order = const_cast<int32_t*>(p.order);
    const int b = threadIdx.x;
    if (b < p.B) {
        const int g = num_graphs == 1 ? 0 : b;
        work[b] = (long long)len.T[b] * p.g.ords[g * 3].total_slots;
    }
    __syncthreads();
    if (b < p.B) {
        int rank = 0;  // sequences that go before this one
        for (int o = 0; o < p.B; ++o) {
            const bool before =
                work[o] != work[b] ? work[o] > work[b]
                                   : (len.T[o] != len.T[b] ? len.T[o] > len.T[b] : o < b);
            rank += before ? 1 : 0;
        }
        order[2 * rank] = b << 1;
        order[2 * rank + 1] = (b << 1) | 1;
    }
    if (b == 0) {
        long long a_at = 0, b_at = 0, s_at = 0;
        for (int i = 0; i < p.B; ++i) {
            const int g = num_graphs == 1 ? 0 : i;
            SeqDesc sd;
            sd.alpha_at = a_at;
            sd.beta_at = b_at;
            sd.T = len.T[i];
            sd.graph = g;
            sd.scal_at = (int32_t)s_at;
            sd.pad = 0;
            seqs[i] = sd;
            a_at += (long long)p.g.ords[g * 3 + 0].num_slices * 64 * (len.T[i] + 1);
            b_at += (long long)p.g.ords[g * 3 + 1].num_slices * 64 * (len.T[i] + 1);
            s_at += len.T[i] + 1;
        }
    }
}
}  // namespace

hipError_t find_static_workspace(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = ptr;
    return hipSuccess;
}

void* static_workspace(int device)
{
    return device >= 0 && device < kMaxDevices ? g_scratch_ptr[device] : nullptr;
}

hipError_t launch_describe(const FbParams& p, const int32_t* lengths, int num_graphs,
                           hipStream_t stream)
{
    if (p.B < 1 || p.B > kStaticMaxBatch) return hipErrorInvalidValue;
    StaticLengths len;
    for (int b = 0; b < kStaticMaxBatch; ++b) len.T[b] = b < p.B ? lengths[b] : 0;
    hipLaunchKernelGGL(k_describe, dim3(1), dim3(kStaticMaxBatch), 0, stream, p, len, num_graphs);
    return hipGetLastError();
}

hipError_t launch_forward_backward(const FbParams& p, const LaunchShape& shape,
                                   hipStream_t stream, hipEvent_t* ev, const Buckets& bk)
{
    return p.wide ? launch_typed<double>(p, shape, stream, ev, bk)
                  : launch_typed<float>(p, shape, stream, ev, bk);
}

}  // namespace lfmmi

#ifdef LFMMI_PHASE_TIMERS
// out[0..8]: clocks per phase of k_occ_planes summed over the workgroups since the
// last reset; out[14]: workgroups, out[15]: frame groups. out[16 + 4 w + q]: clocks of
// phase q of a step in wave w of the register-resident k_rec, out[80]: steps (both
// directions of every sequence). Synchronises the device.
extern "C" int lfmmi_phase_timers_read(unsigned long long out[81], int reset)
{
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    if (hipMemcpyFromSymbol(out, HIP_SYMBOL(lfmmi::g_phase_clocks), sizeof(unsigned long long) * 16) !=
            hipSuccess ||
        hipMemcpyFromSymbol(out + 16, HIP_SYMBOL(lfmmi::g_rec_clocks), sizeof(unsigned long long) * 65) !=
            hipSuccess)
        return 2;
    if (reset) {
        const unsigned long long zero[65] = {};
        if (hipMemcpyToSymbol(HIP_SYMBOL(lfmmi::g_phase_clocks), zero, sizeof(unsigned long long) * 16) !=
                hipSuccess ||
            hipMemcpyToSymbol(HIP_SYMBOL(lfmmi::g_rec_clocks), zero, sizeof zero) != hipSuccess)
            return 3;
    }
    return 0;
}
#endif
