// HIP kernels (gfx950) of the batched LF-MMI forward-backward.
//
// Pipeline of one call (all on the caller's stream):
//   k_emit  e_t[d] = exp(x_t[d] - max_d x_t[d]) for every valid frame, in parallel
//   k_rec   one workgroup per (sequence, direction): the alpha recursion of
//           Algorithm 1 and the mirrored beta recursion, time loop on device,
//           the current vector in LDS, arcs streamed as sliced-ELL records,
//           leaky-HMM mixing and per-frame rescaling fused, scaled trellis rows
//           and per-frame normalisers spilled to HBM
//   k_scan  fp64 prefix sums of the log normalisers: log Z, per-frame occupancy
//           scale, objective and status
//   k_occ   pdf occupancies of Eq. 3 for every frame in parallel and the
//           gradient write
//
// Scaled quantities: alpha'_t = ahat_t * exp(sum_{tau<=t} log n_tau) * (frame
// maxima), likewise beta; the frame maxima cancel in the occupancies and are
// added back into log Z.
#include "kernels.h"

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
    const int b = blockIdx.y;
    if (t >= p.seqs[b].T) return;
    const size_t at = ((size_t)b * p.T + t) * p.P;
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
constexpr int kYRegs = 4;

// One arc slot: w * e[pdf] in fp32, times the gathered state value in Real.
template <typename Real>
__device__ __forceinline__ Real arc_term(const uint2 r, const Real* X, const float* Y)
{
    return (Real)(__uint_as_float(r.y) * lds_at(Y, r.x >> 16)) * lds_at(X, r.x & 0xffffu);
}

// Real = float for graphs whose states are all final (denominator-like: the
// scaled vectors stay within fp32 range), double otherwise (numerator-like
// left-to-right graphs, where the states that matter can hold a fraction of the
// frame's mass far below 1e-38).
template <typename Real>
__global__ void __launch_bounds__(1024) k_rec(FbParams p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x;
    const int nwaves = nthreads >> 6;
    const int code = p.order[blockIdx.x];
    const int b = code >> 1, dir = code & 1;
    const SeqDesc sd = p.seqs[b];
    const OrdDesc od = p.g.ords[sd.graph * 3 + dir];
    const int T = sd.T;
    const int P = p.P;
    const int rows = od.num_slices * 64;
    const int Ppad = (P + 63) & ~63;

    Real* X0 = reinterpret_cast<Real*>(lds_raw);
    Real* X1 = X0 + p.lds_rows;
    Real* part = X1 + p.lds_rows;  // [16][2]
    float* Y0 = reinterpret_cast<float*>(part + 32);
    float* Y1 = Y0 + Ppad;

    Real* trel = static_cast<Real*>(dir == 0 ? p.alpha : p.beta) +
                 (dir == 0 ? sd.alpha_at : sd.beta_at);
    Real* scal = static_cast<Real*>(p.scal) + (size_t)dir * p.scal_total + sd.scal_at;
    const uint2* recs = p.g.recs + (size_t)od.rec_at * 64 + lane;
    const int32_t* so = p.g.slice_off + od.slice_off_at;
    const float* va = p.g.va + od.vec_at;
    const float* vb = p.g.vb + od.vec_at;
    const Real eps = (Real)p.leak;

    int s0 = 0, s1 = 0;
    if (wave < od.num_waves) {
        s0 = p.g.wave_first[od.wave_first_at + wave];
        s1 = p.g.wave_first[od.wave_first_at + wave + 1];
    }
    const size_t erow0 = (size_t)b * p.T;

    // ---- step 0: vhat_0 = leak(init) / sum(init)
    {
        Real n = 0, s = 0;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            const Real v = (Real)p.g.vinit[od.vec_at + row];
            X0[row] = v;
            n += v;
            s += (Real)va[row] * v;
        }
        n = wave_sum(n);
        s = wave_sum(s);
        if (lane == 0) { part[wave * 2] = n; part[wave * 2 + 1] = s; }
        __syncthreads();
        Real N = 0, Sd = 0;
        for (int w = 0; w < nwaves; ++w) { N += part[w * 2]; Sd += part[w * 2 + 1]; }
        const Real inv = N > 0 ? (Real)1 / N : (Real)0;
        const Real c = eps * Sd * inv;
        const int ti = dir == 0 ? 0 : T;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            const Real v = c * (Real)vb[row] + X0[row] * inv;
            X0[row] = v;
            trel[(size_t)ti * rows + row] = v;
        }
        if (tid == 0) scal[ti] = N;
        if (T > 0) {
            const int fr = dir == 0 ? 0 : T - 1;
            const float* e = p.emis + (erow0 + fr) * P;
            for (int d = tid; d < P; d += nthreads) Y0[d] = e[d];
        }
        __syncthreads();
    }

    // ---- steps 1..T
    for (int k = 1; k <= T; ++k) {
        const Real* Xc = (k & 1) ? X0 : X1;
        Real* Xn = (k & 1) ? X1 : X0;
        const float* Yc = (k & 1) ? Y0 : Y1;
        float* Yn = (k & 1) ? Y1 : Y0;

        // emission row of the next step, issued early
        float yreg[kYRegs];
        const bool more = k < T;
        const int frn = dir == 0 ? k : T - k - 1;
        const float* en = p.emis + (erow0 + (more ? frn : 0)) * P;
#pragma unroll
        for (int i = 0; i < kYRegs; ++i) {
            const int d = tid + i * nthreads;
            yreg[i] = (more && d < P) ? en[d] : 0.f;
        }

        Real n = 0, s = 0;
        for (int sl = s0; sl < s1; ++sl) {
            const int o0 = so[sl], o1 = so[sl + 1];
            const uint2* rp = recs + (size_t)o0 * 64;
            Real acc = 0;
            int i = o0;
            for (; i + 4 <= o1; i += 4) {
                const uint2 r0 = rp[0], r1 = rp[64], r2 = rp[128], r3 = rp[192];
                rp += 256;
                acc += arc_term(r0, Xc, Yc);
                acc += arc_term(r1, Xc, Yc);
                acc += arc_term(r2, Xc, Yc);
                acc += arc_term(r3, Xc, Yc);
            }
            for (; i < o1; ++i) {
                acc += arc_term(rp[0], Xc, Yc);
                rp += 64;
            }
            const int row = sl * 64 + lane;
            Xn[row] = acc;
            n += acc;
            s += (Real)va[row] * acc;
        }
        n = wave_sum(n);
        s = wave_sum(s);
        if (lane == 0) { part[wave * 2] = n; part[wave * 2 + 1] = s; }
        __syncthreads();

        Real N = 0, Sd = 0;
        for (int w = 0; w < nwaves; ++w) { N += part[w * 2]; Sd += part[w * 2 + 1]; }
        const Real inv = N > 0 ? (Real)1 / N : (Real)0;
        const Real c = eps * Sd * inv;
        const int ti = dir == 0 ? k : T - k;
        Real* tr = trel + (size_t)ti * rows;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            const Real v = c * (Real)vb[row] + Xn[row] * inv;
            Xn[row] = v;
            tr[row] = v;
        }
        if (tid == 0) scal[ti] = N;
        if (more) {
#pragma unroll
            for (int i = 0; i < kYRegs; ++i) {
                const int d = tid + i * nthreads;
                if (d < P) Yn[d] = yreg[i];
            }
            for (int d = tid + kYRegs * nthreads; d < P; d += nthreads) Yn[d] = en[d];
        }
        __syncthreads();
    }

    // ---- closing dot product: alpha side sum_j f[j] ahat_T[j], beta side sum_i pi[i] bhat_0[i]
    {
        const Real* Xc = (T & 1) ? X1 : X0;
        Real z = 0;
        for (int sl = s0; sl < s1; ++sl) {
            const int row = sl * 64 + lane;
            z += (Real)p.g.vfin[od.vec_at + row] * Xc[row];
        }
        z = wave_sum(z);
        if (lane == 0) part[wave * 2] = z;
        __syncthreads();
        if (tid == 0) {
            Real Z = 0;
            for (int w = 0; w < nwaves; ++w) Z += part[w * 2];
            static_cast<Real*>(p.zfin)[(size_t)dir * p.B + b] = Z;
        }
    }
}

// ---------------------------------------------------------------------------
// Scales: log Z_b = log(zfin) + sum_t log n_t (+ the frame maxima), and the
// factor that turns ahat_{t-1} * w * e_t * bhat_t into an occupancy:
//   c_t = exp(A_{t-1} + B_t - log Z'),  A, B = prefix / suffix sums of log n.
// ---------------------------------------------------------------------------
template <typename Real>
__global__ void __launch_bounds__(256) k_scan(FbParams p)
{
    __shared__ double sa[256], sb[256], sm[256];
    __shared__ double tot[3];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const SeqDesc sd = p.seqs[b];
    const int T = sd.T;
    const int n = T + 1;
    const Real* na = static_cast<const Real*>(p.scal) + sd.scal_at;
    const Real* nb = static_cast<const Real*>(p.scal) + p.scal_total + sd.scal_at;
    Real* cfac = static_cast<Real*>(p.cfac) + sd.scal_at;
    const int chunk = (n + 255) / 256;
    const int i0 = min(tid * chunk, n), i1 = min(i0 + chunk, n);
    double la = 0.0, lb = 0.0, lm = 0.0;
    for (int i = i0; i < i1; ++i) {
        la += log((double)na[i]);
        lb += log((double)nb[i]);
    }
    for (int t = tid; t < T; t += 256) lm += (double)p.rowmax[(size_t)b * p.T + t];
    sa[tid] = la; sb[tid] = lb; sm[tid] = lm;
    __syncthreads();
    if (tid == 0) {
        double ra = 0.0, rb = 0.0, rm = 0.0;
        for (int i = 0; i < 256; ++i) {
            const double xa = sa[i], xb = sb[i];
            sa[i] = ra; sb[i] = rb;  // exclusive prefixes
            ra += xa; rb += xb; rm += sm[i];
        }
        tot[0] = ra; tot[1] = rb; tot[2] = rm;
    }
    __syncthreads();
    const double totB = tot[1], msum = tot[2];
    const double lz = log((double)static_cast<const Real*>(p.zfin)[b]) + tot[0];
    const bool nonfinite_in = !(msum == msum);
    const bool dead = !(lz > -INFINITY && lz < INFINITY) || nonfinite_in;
    double ra = sa[tid], rb = sb[tid];
    for (int i = i0; i < i1; ++i) {
        if (i >= 1) cfac[i] = dead ? (Real)0 : (Real)exp(ra + (totB - rb) - lz);
        ra += log((double)na[i]);
        rb += log((double)nb[i]);
    }
    if (tid == 0) {
        int st = 0;
        if (nonfinite_in) st |= 2;
        if (dead) st |= 1;
        const float val = nonfinite_in ? __builtin_nanf("") : (float)(lz + msum);
        const float out = p.grad_scale * val;
        p.objf[b] = p.accumulate ? p.objf[b] + out : out;
        p.status_ws[b] = st;
        if (p.status_out) p.status_out[b] = p.accumulate ? (p.status_out[b] | st) : st;
    }
}

// ---------------------------------------------------------------------------
// Occupancy and gradient, frames in parallel. Rows of the OCC ordering are
// pieces of one pdf's arc list; a row's sum goes to its pdf's LDS bin.
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
    const int b = blockIdx.y;
    const SeqDesc sd = p.seqs[b];
    const int T = sd.T;
    const int P = p.P;
    const int Ppad = (P + 63) & ~63;
    const OrdDesc od = p.g.ords[sd.graph * 3 + 2];
    const int rows_f = p.g.ords[sd.graph * 3 + 0].num_slices * 64;
    const int rows_b = p.g.ords[sd.graph * 3 + 1].num_slices * 64;

    Real* XA = reinterpret_cast<Real*>(lds_raw);
    Real* XB = XA + p.lds_rows_occ_a;
    Real* bins0 = XB + p.lds_rows_occ_b;
    Real* bins1 = bins0 + Ppad;

    const uint2* recs = p.g.recs + (size_t)od.rec_at * 64 + lane;
    const int32_t* so = p.g.slice_off + od.slice_off_at;
    const int32_t* row_pdf4 = p.g.row_pdf4 + od.vec_at;
    const Real* cfac = static_cast<const Real*>(p.cfac) + sd.scal_at;
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
        Real* bins = (t & 1) ? bins1 : bins0;
        const Real* ar = static_cast<const Real*>(p.alpha) + sd.alpha_at + (size_t)(t - 1) * rows_f;
        const Real* br = static_cast<const Real*>(p.beta) + sd.beta_at + (size_t)t * rows_b;
        for (int r = tid; r < rows_f; r += nthreads) XA[r] = ar[r];
        for (int r = tid; r < rows_b; r += nthreads) XB[r] = br[r];
        for (int d = tid; d < P; d += nthreads) bins[d] = 0;
        __syncthreads();
        for (int sl = s0; sl < s1; ++sl) {
            const int o0 = so[sl], o1 = so[sl + 1];
            const uint2* rp = recs + (size_t)o0 * 64;
            Real acc = 0;
            int i = o0;
            for (; i + 4 <= o1; i += 4) {
                const uint2 r0 = rp[0], r1 = rp[64], r2 = rp[128], r3 = rp[192];
                rp += 256;
                acc += occ_term(r0, XA, XB);
                acc += occ_term(r1, XA, XB);
                acc += occ_term(r2, XA, XB);
                acc += occ_term(r3, XA, XB);
            }
            for (; i < o1; ++i) {
                acc += occ_term(rp[0], XA, XB);
                rp += 64;
            }
            const int pd = row_pdf4[sl * 64 + lane];
            if (pd >= 0) atomicAdd(bins + (pd >> 2), acc);
        }
        __syncthreads();
        const Real scale = (Real)p.grad_scale * c;
        const float* e = p.emis + at;
        for (int d = tid; d < P; d += nthreads) {
            const float v = (float)(scale * (Real)e[d] * bins[d]);
            g[d] = p.accumulate ? g[d] + v : v;
        }
    }
}

}  // namespace

hipError_t configure_kernels()
{
    const void* fns[] = {reinterpret_cast<const void*>(k_rec<float>),
                         reinterpret_cast<const void*>(k_rec<double>),
                         reinterpret_cast<const void*>(k_occ<float>),
                         reinterpret_cast<const void*>(k_occ<double>)};
    for (const void* f : fns) {
        hipError_t e =
            hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

size_t rec_lds_bytes(int lds_rows, int P, bool wide)
{
    const size_t Ppad = (size_t)((P + 63) & ~63);
    return (2 * (size_t)lds_rows + 32) * (wide ? 8 : 4) + 2 * Ppad * 4;
}

size_t occ_lds_bytes(int rows_a, int rows_b, int P, bool wide)
{
    const size_t Ppad = (size_t)((P + 63) & ~63);
    return ((size_t)rows_a + rows_b + 2 * Ppad) * (wide ? 8 : 4);
}

template <typename Real>
static hipError_t launch_typed(const FbParams& p, const LaunchShape& shape, hipStream_t stream,
                               hipEvent_t* ev)
{
    hipError_t e;
    const bool wide = sizeof(Real) == 8;
#define LFMMI_EV(i)                                                   \
    if (ev) { e = hipEventRecord(ev[i], stream); if (e != hipSuccess) return e; }
    LFMMI_EV(0)
    if (p.T > 0) {
        dim3 grid((p.T + 3) / 4, p.B);
        hipLaunchKernelGGL(k_emit, grid, dim3(256), 0, stream, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    LFMMI_EV(1)
    hipLaunchKernelGGL(k_rec<Real>, dim3(2 * p.B), dim3(shape.rec_threads),
                       rec_lds_bytes(p.lds_rows, p.P, wide), stream, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    LFMMI_EV(2)
    hipLaunchKernelGGL(k_scan<Real>, dim3(p.B), dim3(256), 0, stream, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    LFMMI_EV(3)
    if (p.T > 0) {
        dim3 grid((p.T + shape.occ_frames - 1) / shape.occ_frames, p.B);
        hipLaunchKernelGGL(k_occ<Real>, grid, dim3(shape.occ_threads),
                           occ_lds_bytes(p.lds_rows_occ_a, p.lds_rows_occ_b, p.P, wide), stream,
                           p, shape.occ_frames);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    LFMMI_EV(4)
#undef LFMMI_EV
    return hipSuccess;
}

hipError_t launch_forward_backward(const FbParams& p, const LaunchShape& shape,
                                   hipStream_t stream, hipEvent_t* ev)
{
    return p.wide ? launch_typed<double>(p, shape, stream, ev)
                  : launch_typed<float>(p, shape, stream, ev);
}

}  // namespace lfmmi
