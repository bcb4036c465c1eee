// Microbenchmarks behind the roofline numbers of the LF-MMI recursion (gfx950).
//
//   lfmmi_microbench lds        LDS read bandwidth: conflict-free 4-byte reads, 8- and
//                               16-byte reads, random 4-byte gathers; one workgroup on
//                               one compute unit, then every compute unit at once; the
//                               shader clock under that load
//   lfmmi_microbench exchange   what it costs two workgroups on different compute units
//                               to hand each other a vector once per step through device
//                               memory (the per-frame exchange a recursion split over
//                               several compute units would need): same XCD (one L2)
//                               and different XCDs, several protocols
//   lfmmi_microbench cluster    the same for 2 or 4 workgroups that keep a 5,056-row state
//                               vector between them, with a stand-in for their work
//
// Every wait in the exchange kernels is bounded: a workgroup that does not see its
// partner within kSpinLimit polls sets an error flag and both leave the loop, so
// every wave reaches the end of its kernel whatever the placement.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define CK(x)                                                                        \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

typedef __attribute__((address_space(3))) float lds_float_t;
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x2_t lds_float2_t;
typedef __attribute__((address_space(3))) f32x4_t lds_float4_t;

__device__ __forceinline__ float lds_ld(uint32_t a)
{
    return *reinterpret_cast<const lds_float_t*>(static_cast<uintptr_t>(a));
}
__device__ __forceinline__ f32x2_t lds_ld2(uint32_t a)
{
    return *reinterpret_cast<const lds_float2_t*>(static_cast<uintptr_t>(a));
}
__device__ __forceinline__ f32x4_t lds_ld4(uint32_t a)
{
    return *reinterpret_cast<const lds_float4_t*>(static_cast<uintptr_t>(a));
}
__device__ __forceinline__ void lds_st(uint32_t a, float v)
{
    *reinterpret_cast<lds_float_t*>(static_cast<uintptr_t>(a)) = v;
}

// ---------------------------------------------------------------------------
// LDS read streams. 64 KB of dynamic LDS (the kernel declares no static LDS, so
// it starts at address 0); a lane reads at its own base address plus immediates,
// 16 reads per loop trip, the sum kept so that nothing is optimised away.
// W = bytes per lane and read (4, 8, 16).
// ---------------------------------------------------------------------------
template <int W>
__global__ void __launch_bounds__(1024) k_lds_read(const uint32_t* base_of_thread, float* out,
                                                   long long* clocks, int trips)
{
    extern __shared__ float lds_dyn[];
    const int tid = threadIdx.x;
    for (int i = tid; i < 16384; i += blockDim.x) lds_st((uint32_t)i * 4u, (float)i * 1e-6f);
    __syncthreads();
    const uint32_t base = base_of_thread[tid];  // byte address below 32 KB, multiple of W
    float acc = 0.f;
    const long long c0 = clock64();
    const long long w0 = wall_clock64();
    for (int it = 0; it < trips; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            // + u * 2 KB: the same banks again, other words
            const uint32_t a = base + (uint32_t)u * 2048u;
            if constexpr (W == 4) {
                acc += lds_ld(a);
            } else if constexpr (W == 8) {
                const f32x2_t v = lds_ld2(a);
                acc += v.x + v.y;
            } else {
                const f32x4_t v = lds_ld4(a);
                acc += v.x + v.y + v.z + v.w;
            }
        }
        asm volatile("" : "+v"(acc));
    }
    const long long c1 = clock64();
    const long long w1 = wall_clock64();
    out[(size_t)blockIdx.x * blockDim.x + tid] = acc;
    // per wave: where its loop began and ended on the shader clock and on the 100 MHz
    // wall clock (a compute unit serves its oldest waves first, so one wave's span
    // says little: the workgroup's loop runs from the first start to the last end)
    if ((tid & 63) == 0) {
        long long* c = clocks + ((size_t)blockIdx.x * 16 + (tid >> 6)) * 4;
        c[0] = c0;
        c[1] = c1;
        c[2] = w0;
        c[3] = w1;
    }
}

struct Pattern {
    const char* name;
    int width;  // bytes per lane
    int kind;   // 0: lane * width (conflict-free), 1: random word, 2: random of 84 words
};

static void run_lds(int device)
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, device));
    const int cus = prop.multiProcessorCount;
    std::printf("device %s, %d compute units, clockRate %d kHz, wall clock %d kHz\n", prop.gcnArchName,
                cus, prop.clockRate, 100000);
    const int threads = 1024, trips = 4000;
    uint32_t* d_base;
    float* d_out;
    long long* d_clk;
    const int max_blocks = 2 * cus;
    CK(hipMalloc(&d_base, threads * 4));
    CK(hipMalloc(&d_out, (size_t)max_blocks * threads * 4));
    CK(hipMalloc(&d_clk, (size_t)max_blocks * 16 * 4 * 8));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const Pattern pats[] = {
        {"4-byte reads, lane l reads word l (conflict-free)", 4, 0},
        {"4-byte reads, random words (gather)", 4, 1},
        {"4-byte reads, random among 84 words", 4, 2},
        {"8-byte reads, consecutive", 8, 0},
        {"16-byte reads, consecutive", 16, 0},
    };
    std::printf("%-52s %6s %12s %12s %10s %12s\n", "pattern", "WGs", "clk/wave-rd", "B/clk/CU", "GHz",
                "chip TB/s");
    for (const Pattern& p : pats) {
        std::vector<uint32_t> base(threads);
        std::srand(1);
        for (int t = 0; t < threads; ++t) {
            const int lane = t & 63;
            uint32_t word;
            if (p.kind == 0) word = (uint32_t)lane * (p.width / 4);
            else if (p.kind == 1) word = (uint32_t)(std::rand() % 512);
            else word = (uint32_t)(std::rand() % 84);
            base[t] = word * 4u;  // + 15 * 2 KB + 16 bytes stays below 64 KB
        }
        CK(hipMemcpy(d_base, base.data(), threads * 4, hipMemcpyHostToDevice));
        for (int blocks : {1, cus, 2 * cus}) {
            auto launch = [&](int n) {
                if (p.width == 4)
                    hipLaunchKernelGGL(k_lds_read<4>, dim3(blocks), dim3(threads), 65536, 0, d_base, d_out, d_clk, n);
                else if (p.width == 8)
                    hipLaunchKernelGGL(k_lds_read<8>, dim3(blocks), dim3(threads), 65536, 0, d_base, d_out, d_clk, n);
                else
                    hipLaunchKernelGGL(k_lds_read<16>, dim3(blocks), dim3(threads), 65536, 0, d_base, d_out, d_clk, n);
                CK(hipGetLastError());
            };
            launch(50);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            launch(trips);
            CK(hipEventRecord(e1));
            CK(hipDeviceSynchronize());
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            std::vector<long long> clk((size_t)blocks * 16 * 4);
            CK(hipMemcpy(clk.data(), d_clk, clk.size() * 8, hipMemcpyDeviceToHost));
            double csum = 0, wsum = 0;  // per workgroup: first start to last end
            for (int b = 0; b < blocks; ++b) {
                long long c_lo = clk[(size_t)b * 64], c_hi = clk[(size_t)b * 64 + 1];
                long long w_lo = clk[(size_t)b * 64 + 2], w_hi = clk[(size_t)b * 64 + 3];
                for (int w = 1; w < threads / 64; ++w) {
                    const long long* c = &clk[((size_t)b * 16 + w) * 4];
                    c_lo = std::min(c_lo, c[0]);
                    c_hi = std::max(c_hi, c[1]);
                    w_lo = std::min(w_lo, c[2]);
                    w_hi = std::max(w_hi, c[3]);
                }
                csum += (double)(c_hi - c_lo);
                wsum += (double)(w_hi - w_lo);
            }
            const double wave_reads = (double)trips * 16 * (threads / 64);  // per workgroup
            const double clk_per_read = csum / blocks / wave_reads;
            const double ghz = csum / wsum * 0.1;  // shader clocks per 100 MHz tick
            const double bytes = (double)blocks * wave_reads * 64 * p.width;
            // a compute unit holds one of these workgroups at a time (64 KB LDS, 1024 threads)
            const double per_cu = 64.0 * p.width / clk_per_read;
            std::printf("%-52s %6d %12.2f %12.1f %10.2f %12.2f\n", p.name, blocks, clk_per_read, per_cu,
                        ghz, bytes / (ms * 1e-3) / 1e12);
            std::fflush(stdout);
        }
    }
    CK(hipFree(d_base));
    CK(hipFree(d_out));
    CK(hipFree(d_clk));
}

// ---------------------------------------------------------------------------
// Exchange between two workgroups. Of a grid of 16 workgroups only `wg_a` and
// `wg_b` take part (workgroup ids are dealt to the XCDs round robin, so ids that
// are congruent mod 8 share an XCD and its L2; the kernel also records the XCC id
// each of the two ran on). Each step both write a vector of `lanes` values for the
// partner and read the partner's, double buffered: a workgroup starts step k + 1
// only after it has read the partner's step-k vector, which the partner wrote
// after reading step k - 1, so a buffer is never overwritten before it is read.
//
// MODE 0: payload by plain stores, agent-scope release fence, flag store; the
//         reader polls the flag, agent-scope acquire fence, plain loads (what the
//         language memory model asks for between any two workgroups).
// MODE 1: payload and flag by relaxed agent-scope atomic stores / loads (they go to
//         L2 and are read from L2, no write-back or invalidate of the L2), ordered
//         by waiting for the payload stores and a workgroup barrier before the flag.
// MODE 2: no flag: every 8-byte payload word carries the step number next to its
//         value, written by one relaxed agent-scope atomic store and polled by
//         the lane that needs it.
// ---------------------------------------------------------------------------
constexpr int kSpinLimit = 1 << 18;

struct ExchangeBuffers {
    unsigned long long* payload;  // [2 workgroups][2 parities][1024] {step << 32 | value bits}
    unsigned int* flag;           // [2 workgroups][64] (one flag per workgroup, padded)
    unsigned int* info;           // [0] error count, [1..2] XCC id of a / b, [3..4] HW_ID, [5] bad values
    long long* clocks;            // [2][2] shader clocks, wall clocks of the loop
};

template <int MODE>
__global__ void __launch_bounds__(1024) k_exchange(ExchangeBuffers x, int wg_a, int wg_b, int lanes,
                                                   int steps)
{
    const int me = (int)blockIdx.x == wg_a ? 0 : ((int)blockIdx.x == wg_b ? 1 : -1);
    if (me < 0) return;
    const int tid = threadIdx.x;
    if (tid == 0) {
        // XCC_ID (hardware register 20, bits 3:0) and HW_ID (register 4)
        x.info[1 + me] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
        x.info[3 + me] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
    }
    unsigned long long* mine = x.payload + (size_t)me * 2 * 1024;
    unsigned long long* theirs = x.payload + (size_t)(1 - me) * 2 * 1024;
    unsigned int* my_flag = x.flag + me * 64;
    unsigned int* their_flag = x.flag + (1 - me) * 64;
    int my_stop = 0, stop = 0;  // a wait that ran out; agreed on at a barrier of every step
    float carry = 1.0f + (float)tid * 1e-3f;
    int bad = 0;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int k = 1; k <= steps; ++k) {
        const int par = k & 1;
        const float send = carry + (float)me;
        if constexpr (MODE == 0) {
            if (tid < lanes) mine[par * 1024 + tid] = (unsigned long long)__float_as_uint(send);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __syncthreads();
            if (tid == 0) {
                __hip_atomic_store(my_flag, (unsigned)k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                int spins = 0;
                while (__hip_atomic_load(their_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)k)
                    if (++spins > kSpinLimit) { my_stop = 1; break; }
            }
            stop = __syncthreads_or(my_stop);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            if (tid < lanes) {
                const float got = __uint_as_float((unsigned)theirs[par * 1024 + tid]);
                bad += (!(stop | my_stop) && got != carry + (float)(1 - me)) ? 1 : 0;
                carry = got * 0.5f + send * 0.5f;
            }
        } else if constexpr (MODE == 1) {
            if (tid < lanes)
                __hip_atomic_store(mine + par * 1024 + tid, (unsigned long long)__float_as_uint(send),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // waits for the stores
            __syncthreads();
            if (tid == 0) {
                __hip_atomic_store(my_flag, (unsigned)k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                int spins = 0;
                while (__hip_atomic_load(their_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)k)
                    if (++spins > kSpinLimit) { my_stop = 1; break; }
            }
            stop = __syncthreads_or(my_stop);
            if (tid < lanes) {
                const unsigned long long v = __hip_atomic_load(theirs + par * 1024 + tid, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                const float got = __uint_as_float((unsigned)v);
                bad += (!(stop | my_stop) && got != carry + (float)(1 - me)) ? 1 : 0;
                carry = got * 0.5f + send * 0.5f;
            }
        } else {
            if (tid < lanes) {
                const unsigned long long word =
                    ((unsigned long long)(unsigned)k << 32) | __float_as_uint(send);
                __hip_atomic_store(mine + par * 1024 + tid, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                unsigned long long v;
                int spins = 0;
                while (true) {
                    v = __hip_atomic_load(theirs + par * 1024 + tid, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
                    if ((unsigned)(v >> 32) == (unsigned)k) break;
                    if (++spins > kSpinLimit) { my_stop = 1; break; }
                }
                const float got = __uint_as_float((unsigned)v);
                bad += (!(stop | my_stop) && got != carry + (float)(1 - me)) ? 1 : 0;
                carry = got * 0.5f + send * 0.5f;
            }
            // the state vector of a recursion step is complete only when every lane has
            // its values: one workgroup barrier per step, as in the real kernel
            stop = __syncthreads_or(my_stop);
        }
        if (stop) break;  // workgroup-uniform: the barrier's own result
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (tid == 0) {
        x.clocks[me * 2] = c1 - c0;
        x.clocks[me * 2 + 1] = w1 - w0;
        if (stop) atomicAdd(x.info, 1u);
    }
    if (bad) atomicAdd(x.info + 5, (unsigned)bad);
}

static void run_exchange()
{
    ExchangeBuffers x;
    CK(hipMalloc(&x.payload, 2 * 2 * 1024 * 8));
    CK(hipMalloc(&x.flag, 2 * 64 * 4));
    CK(hipMalloc(&x.info, 8 * 4));
    CK(hipMalloc(&x.clocks, 4 * 8));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int steps = 20000;
    const char* modes[] = {"agent-scope release / acquire fences + flag",
                           "relaxed agent-scope atomics (L2), barrier, flag",
                           "step number inside every 8-byte word, no flag"};
    std::printf("%-50s %-10s %6s %10s %8s %8s %6s %6s\n", "protocol", "workgroups", "lanes", "ns/step",
                "xcc a", "xcc b", "stuck", "bad");
    for (int mode = 0; mode < 3; ++mode)
        for (int pair = 0; pair < 3; ++pair)
            for (int lanes : {1, 1024}) {
                const int wg_a = 0, wg_b = pair == 0 ? 8 : (pair == 1 ? 1 : 4);
                CK(hipMemset(x.payload, 0, 2 * 2 * 1024 * 8));
                CK(hipMemset(x.flag, 0, 2 * 64 * 4));
                CK(hipMemset(x.info, 0, 8 * 4));
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(e0));
                if (mode == 0)
                    hipLaunchKernelGGL(k_exchange<0>, dim3(16), dim3(1024), 0, 0, x, wg_a, wg_b, lanes, steps);
                else if (mode == 1)
                    hipLaunchKernelGGL(k_exchange<1>, dim3(16), dim3(1024), 0, 0, x, wg_a, wg_b, lanes, steps);
                else
                    hipLaunchKernelGGL(k_exchange<2>, dim3(16), dim3(1024), 0, 0, x, wg_a, wg_b, lanes, steps);
                CK(hipGetLastError());
                CK(hipEventRecord(e1));
                CK(hipDeviceSynchronize());
                float ms;
                CK(hipEventElapsedTime(&ms, e0, e1));
                unsigned info[8];
                CK(hipMemcpy(info, x.info, sizeof(info), hipMemcpyDeviceToHost));
                char who[32];
                std::snprintf(who, sizeof(who), "%d and %d", wg_a, wg_b);
                std::printf("%-50s %-10s %6d %10.0f %8u %8u %6u %6u\n", modes[mode], who, lanes,
                            ms * 1e6 / steps, info[1], info[2], info[0], info[5]);
                std::fflush(stdout);
            }
    CK(hipFree(x.payload));
    CK(hipFree(x.flag));
    CK(hipFree(x.info));
    CK(hipFree(x.clocks));
}

// ---------------------------------------------------------------------------
// A cluster of C workgroups that keep one state vector of `rows` values between
// them, as a recursion split over C compute units would: each step every member
// publishes its share of the rows (rows / C values, 8-byte words that carry the
// step number, relaxed agent-scope atomic stores) and imports everybody else's
// (polling each word until its step number is there), writes them into its LDS,
// and meets at a workgroup barrier; `work` dependent multiply-adds per thread stand
// for the member's share of the recursion step. Members are workgroups
// first, first + stride, ...: stride 8 keeps a cluster inside one XCD.
// ---------------------------------------------------------------------------
struct ClusterBuffers {
    unsigned long long* rows;  // [clusters][2 parities][rows]
    unsigned int* info;        // [0] waits that ran out, [1] wrong values
};

__global__ void __launch_bounds__(1024) k_cluster(ClusterBuffers x, int C, int stride, int rows,
                                                  int steps, int work, int clusters)
{
    extern __shared__ float lds_dyn[];
    // workgroup id -> (cluster, member): cluster c holds ids c % stride + stride * (C * (c / stride) + m)
    const int id = blockIdx.x;
    const int lane_of = id % stride, group = id / stride;
    const int member = group % C, cluster = (group / C) * stride + lane_of;
    if (cluster >= clusters) return;
    const int tid = threadIdx.x;
    const int share = (rows + C - 1) / C;
    const int own0 = member * share, own1 = min(own0 + share, rows);
    unsigned long long* buf = x.rows + (size_t)cluster * 2 * rows;
    int my_stop = 0, stop = 0, bad = 0;
    float carry = 1.0f;
    for (int k = 1; k <= steps; ++k) {
        unsigned long long* cur = buf + (size_t)(k & 1) * rows;
        // the member's share of the step
        float acc = carry;
        for (int u = 0; u < work; ++u) {
            acc = fmaf(acc, 0.999f, 0.001f);
            asm volatile("" : "+v"(acc));
        }
        carry = acc;
        // publish own rows: value = row + step (checked by the importers)
        for (int r = own0 + tid; r < own1; r += blockDim.x) {
            const float v = (float)(r + k);
            __hip_atomic_store(cur + r, ((unsigned long long)(unsigned)k << 32) | __float_as_uint(v),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lds_st((uint32_t)r * 4u, v);
        }
        // import the others' rows: up to 8 per thread in flight, polled until all are there
        for (int r0 = tid; r0 < rows; r0 += 8 * blockDim.x) {
            unsigned pending = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = r0 + u * blockDim.x;
                if (r < rows && (r < own0 || r >= own1)) pending |= 1u << u;
            }
            int spins = 0;
            while (pending) {
                unsigned long long w[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (pending & (1u << u))
                        w[u] = __hip_atomic_load(cur + r0 + u * blockDim.x, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if ((pending & (1u << u)) && (unsigned)(w[u] >> 32) == (unsigned)k) {
                        const int r = r0 + u * blockDim.x;
                        const float v = __uint_as_float((unsigned)w[u]);
                        bad += v != (float)(r + k);
                        lds_st((uint32_t)r * 4u, v);
                        pending &= ~(1u << u);
                    }
                if (pending && ++spins > kSpinLimit) {
                    my_stop = 1;
                    break;
                }
            }
        }
        stop = __syncthreads_or(my_stop);
        if (stop) break;
    }
    if (tid == 0 && stop) atomicAdd(x.info, 1u);
    if (bad) atomicAdd(x.info + 1, (unsigned)bad);
    if (tid == 0) lds_dyn[0] = carry;  // keeps the arithmetic
}

static void run_cluster()
{
    const int rows = 5056;  // the 5,000-state graph's padded rows
    const int max_clusters = 64;
    ClusterBuffers x;
    CK(hipMalloc(&x.rows, (size_t)max_clusters * 2 * rows * 8));
    CK(hipMalloc(&x.info, 8 * 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int steps = 4000;
    std::printf("%-10s %-8s %-8s %-9s %-8s %10s %6s %6s\n", "clusters", "members", "stride", "rows", "work",
                "ns/step", "stuck", "bad");
    for (int clusters : {1, 16, 64})
        for (int C : {2, 4})
            for (int stride : {8, 1})
                for (int work : {0, 400}) {
                    if (clusters * C > 256) continue;
                    CK(hipMemset(x.rows, 0, (size_t)max_clusters * 2 * rows * 8));
                    CK(hipMemset(x.info, 0, 8 * 4));
                    // a grid that covers whole groups of `stride` clusters
                    const int groups = (clusters + stride - 1) / stride;
                    const int grid = groups * C * stride;
                    CK(hipDeviceSynchronize());
                    CK(hipEventRecord(e0));
                    hipLaunchKernelGGL(k_cluster, dim3(grid), dim3(1024), 32768, 0, x, C, stride, rows, steps,
                                       work, clusters);
                    CK(hipGetLastError());
                    CK(hipEventRecord(e1));
                    CK(hipDeviceSynchronize());
                    float ms;
                    CK(hipEventElapsedTime(&ms, e0, e1));
                    unsigned info[8];
                    CK(hipMemcpy(info, x.info, sizeof(info), hipMemcpyDeviceToHost));
                    std::printf("%-10d %-8d %-8d %-9d %-8d %10.0f %6u %6u\n", clusters, C, stride, rows, work,
                                ms * 1e6 / steps, info[0], info[1]);
                    std::fflush(stdout);
                }
    CK(hipFree(x.rows));
    CK(hipFree(x.info));
}

int main(int argc, char** argv)
{
    const char* what = argc > 1 ? argv[1] : "all";
    CK(hipSetDevice(0));
    if (!std::strcmp(what, "lds") || !std::strcmp(what, "all")) run_lds(0);
    if (!std::strcmp(what, "exchange") || !std::strcmp(what, "all")) run_exchange();
    if (!std::strcmp(what, "cluster") || !std::strcmp(what, "all")) run_cluster();
    return 0;
}
