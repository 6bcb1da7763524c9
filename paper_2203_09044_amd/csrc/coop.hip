// User side of Algorithm 1 with every gradient read once: the exponent anchor of a user needs the
// largest magnitude of the whole vector before the first element can be converted, so a pass of its
// own over g reads 4 of the path's 16 bytes per element a second time.  Here one resident grid (one
// workgroup of 512 lanes per compute unit) holds a user's whole gradient in registers between the two
// uses: every workgroup owns the same contiguous 1/G of each user's vector, loads its part of g, takes
// the largest magnitude, exchanges it with the other workgroups through one word per workgroup in
// global memory, and converts from registers.  While user u is converted, each register that has been
// consumed is refilled with user u+1's gradient, so the exchange for u+1 starts when u ends.
//
// The exchange uses no fences: a workgroup publishes one self-validating 32-bit word (valid bit |
// magnitude bits) with a relaxed device-scope store, and one wavefront of every workgroup polls the G
// words with relaxed device-scope loads until all are valid.  Nothing else is communicated inside the
// kernel, so no cache needs flushing.  Every wait is bounded: after `spin_limit` polls the workgroup
// raises CO3_ETIMEOUT and goes on with the anchor at its lower clamp (results are then unspecified, but
// in bounds, and the grid drains).
#include "co3_dev.h"
#include "kernels.h"

#define CP_BLOCK 512
#define CP_WAVES (CP_BLOCK / CO3_WAVE)
#define CP_VEC 4
#define CP_STEP (CO3_WAVE * CP_VEC)          // elements that one load of a wavefront covers: one KiB
#define CP_KPT_MAX CO3_COOP_KPT_MAX          // steps per lane: 16-byte pieces of g that a lane keeps in registers
#ifndef CP_AHEAD
#define CP_AHEAD 6                           // memory loads in flight per lane ahead of the conversion
#endif
#ifdef CP_MAP_BLOCK
#define CP_RUN_STRIDE (CP_WAVES * CP_STEP)
#else
#define CP_RUN_STRIDE CP_STEP
#endif
#define CP_HIST_SLOTS 1024                   // LDS counters per wavefront
#define CP_VALID 0x80000000u

__device__ __forceinline__ uint32_t ld_relaxed_agent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed_agent(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t absbits4(float4 v, uint32_t m)
{
    uint32_t a0 = __float_as_uint(v.x) & 0x7fffffffu, a1 = __float_as_uint(v.y) & 0x7fffffffu;
    uint32_t a2 = __float_as_uint(v.z) & 0x7fffffffu, a3 = __float_as_uint(v.w) & 0x7fffffffu;
    a0 = a0 > a1 ? a0 : a1;
    a2 = a2 > a3 ? a2 : a3;
    a0 = a0 > a2 ? a0 : a2;
    return m > a0 ? m : a0;
}

// The lane's 4 consecutive floats of a run of 256 that starts at `run` (wavefront-uniform pointer); `rem`
// (uniform) elements of the run lie below n, the others read as +0.  lane4 = 4 * lane.
__device__ __forceinline__ float4 ld4_run(const float *run, int64_t rem, uint32_t lane4)
{
    if (rem >= CP_STEP) return ld_stream_f4(run + lane4);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    const int64_t r = rem - (int64_t)lane4;
    if (r > 0) v.x = run[lane4 + 0];
    if (r > 1) v.y = run[lane4 + 1];
    if (r > 2) v.z = run[lane4 + 2];
    if (r > 3) v.w = run[lane4 + 3];
    return v;
}

// The workgroup's largest magnitude pattern -> its slot of the row (valid bit set).
__device__ __forceinline__ void coop_publish_max(uint32_t m, uint32_t *row, uint32_t *red)
{
    m = wave_max_u32(m);
    if ((threadIdx.x & (CO3_WAVE - 1)) == 0) red[threadIdx.x / CO3_WAVE] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t mm = red[0];
#pragma unroll
        for (int w = 1; w < CP_WAVES; ++w) mm = mm > red[w] ? mm : red[w];
        st_relaxed_agent(row + blockIdx.x, CP_VALID | mm);
    }
}

// Waits (bounded) until every workgroup's slot of the row is valid; returns the largest magnitude
// pattern over all of them to every lane of the workgroup.
__device__ __forceinline__ uint32_t coop_collect_max(const uint32_t *row, int G, uint32_t spin_limit, uint32_t *red,
                                                     int32_t *status)
{
    if (threadIdx.x < CO3_WAVE) {
        const int lane = threadIdx.x;
        uint32_t m = 0, polls = 0;
        bool done = false;
        while (!done && polls < spin_limit) {
            bool all = true;
            m = 0;
            for (int j = lane; j < G; j += CO3_WAVE) {
                const uint32_t v = ld_relaxed_agent(row + j);
                all &= (v & CP_VALID) != 0u;
                const uint32_t a = v & ~CP_VALID;
                m = m > a ? m : a;
            }
            done = __all(all);
            ++polls;
            if (!done) __builtin_amdgcn_s_sleep(1);
        }
        m = wave_max_u32(m);
        if (lane == 0) {
            if (!done) {
                co3_raise(status, CO3_ETIMEOUT);
                m = 0;
            }
            red[CP_WAVES] = m;
        }
    }
    __syncthreads();
    const uint32_t r = red[CP_WAVES];
    __syncthreads();          // red is reused by the next exchange
    return r;
}

// One user's conversion by one wavefront: KPT runs of 256 elements, the gradient from registers, the memory
// streamed CP_AHEAD runs ahead; as soon as a run is converted its registers take the next user's gradient.
// FULL: all KPT runs lie below n (straight-line code: the compiler can count the memory operations in
// flight exactly); else every access is guarded.  `left` = n - (first element of the wavefront's run 0).
struct CoopWave {
    float *eu;                 // the user's memory at the wavefront's run 0
    uint8_t *su;               // its symbols there, or NULL
    const float *gnext;        // the next user's gradient there (read when `more`)
    bool more;
    int64_t left;
    uint32_t lane4;
    int A, e_min, E, M, codemax;
    float gamma;
    uint32_t *myhist;
    int copies, mycopy;
};

template <int KPT, bool HIST, bool FULL>
__device__ __forceinline__ void coop_convert_user(const CoopWave &w, float4 (&gr)[KPT], float4 (&ev)[CP_AHEAD])
{
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        const int64_t rem = w.left - (int64_t)k * CP_RUN_STRIDE;            // uniform: elements of this run below n
        float *ek = w.eu + k * CP_RUN_STRIDE;
        const float4 gv = gr[k], e4 = ev[k % CP_AHEAD];
        if (k + CP_AHEAD < KPT)
            ev[k % CP_AHEAD] = FULL ? ld_stream_f4(ek + CP_AHEAD * CP_RUN_STRIDE + w.lane4)
                                    : ld4_run(ek + CP_AHEAD * CP_RUN_STRIDE, rem - CP_AHEAD * CP_RUN_STRIDE, w.lane4);
        const float ga[CP_VEC] = {gv.x, gv.y, gv.z, gv.w}, ea[CP_VEC] = {e4.x, e4.y, e4.z, e4.w};
        float en[CP_VEC];
        uint32_t q[CP_VEC];
#pragma unroll
        for (int c = 0; c < CP_VEC; ++c) {
            const float x = ga[c] + w.gamma * ea[c];              // no contraction (build flag): one rounding per operation
            float v;
#ifdef CP_NO_QUANT
            q[c] = __float_as_uint(x) >> 28; v = x * 0.5f;
#else
            co3_quantize(x, w.e_min, w.A, w.E, w.M, w.codemax, q[c], v);
#endif
            en[c] = x - v;
        }
        if (FULL || rem >= CP_STEP) {                             // uniform: the whole run exists
            st_stream_f4(ek + w.lane4, make_float4(en[0], en[1], en[2], en[3]));
#ifndef CP_NO_SYM
            if (w.su)
                *reinterpret_cast<uint32_t *>(w.su + k * CP_RUN_STRIDE + w.lane4) = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
#endif
#ifndef CP_NO_HIST_ATOMICS
            if (HIST) {
#pragma unroll
                for (int c = 0; c < CP_VEC; ++c) atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
            }
#endif
        } else {
#pragma unroll
            for (int c = 0; c < CP_VEC; ++c)
                if ((int64_t)(w.lane4 + c) < rem) {
                    ek[w.lane4 + c] = en[c];
                    if (w.su) w.su[k * CP_RUN_STRIDE + w.lane4 + c] = (uint8_t)q[c];
                    if (HIST) atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
                }
        }
        // the registers are free: the next user's gradient moves in
#ifndef CP_NO_REFILL
        if (w.more)
#else
        if (false)
#endif
            gr[k] = FULL ? ld_stream_f4(w.gnext + k * CP_RUN_STRIDE + w.lane4) : ld4_run(w.gnext + k * CP_RUN_STRIDE, rem, w.lane4);
    }
}

// grid: G workgroups (at most one per compute unit, all resident); workgroup w owns elements
// [w * KPT * 2048, (w + 1) * KPT * 2048) of every user, wavefront v of it the v-th eighth, lane l of the
// wavefront elements 4l .. 4l+3 of each of the wavefront's KPT runs of 256.
template <int KPT, bool HIST>
__global__ __launch_bounds__(CP_BLOCK) void k_coop_convert(const float *__restrict__ g, float *__restrict__ err,
                                                            uint8_t *__restrict__ sym, int64_t n, int64_t stride, int U,
                                                            int32_t *__restrict__ anchor, float gamma,
                                                            co3_fmt fmt, uint32_t *__restrict__ counts,
                                                            uint32_t *__restrict__ slots, uint32_t spin_limit,
                                                            int32_t *status)
{
    const FmtC fc(fmt);
    const int F = fc.F, K = fc.K;
    const int G = gridDim.x;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / CO3_WAVE);     // uniform: addresses of a run are scalar
    __shared__ uint32_t red[CP_WAVES + 1];
    __shared__ uint32_t hist[HIST ? CP_WAVES * CP_HIST_SLOTS : 1];
    const int copies = CP_HIST_SLOTS / K > 32 ? 32 : CP_HIST_SLOTS / K;
    if (HIST) {
        for (int j = threadIdx.x; j < CP_WAVES * CP_HIST_SLOTS; j += CP_BLOCK) hist[j] = 0u;
    }

    // first element of the wavefront's run 0 (uniform); run k lies k * CP_RUN_STRIDE further
#ifdef CP_MAP_BLOCK
    const int64_t first = ((int64_t)blockIdx.x * KPT) * CP_RUN_STRIDE + wave * CP_STEP;
#else
    const int64_t first = (((int64_t)blockIdx.x * CP_WAVES + wave) * KPT) * CP_STEP;
#endif
    const uint32_t lane4 = (uint32_t)lane * CP_VEC;
    const bool full = first + (int64_t)(KPT - 1) * CP_RUN_STRIDE + CP_STEP <= n;      // uniform: every run of the wavefront is whole

    // user 0's gradient: every load of the lane in flight at once
    float4 gr[KPT];
    if (full) {
#pragma unroll
        for (int k = 0; k < KPT; ++k) gr[k] = ld_stream_f4(g + first + k * CP_RUN_STRIDE + lane4);
    } else {
#pragma unroll
        for (int k = 0; k < KPT; ++k) gr[k] = ld4_run(g + first + k * CP_RUN_STRIDE, n - first - k * CP_RUN_STRIDE, lane4);
    }
    {
        uint32_t m = 0;
#pragma unroll
        for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
        coop_publish_max(m, slots, red);
    }

    CoopWave w;
    w.left = n - first;
    w.lane4 = lane4;
    w.E = fc.E;
    w.M = fc.M;
    w.codemax = fc.codemax;
    w.gamma = gamma;
    w.myhist = hist + wave * CP_HIST_SLOTS;
    w.copies = copies;
    w.mycopy = lane & (copies - 1);
    for (int u = 0; u < U; ++u) {
        w.gnext = g + (int64_t)(u + 1) * stride + first;          // only read when u + 1 < U
        w.eu = err + (int64_t)u * stride + first;
        w.su = sym ? sym + (int64_t)u * stride + first : nullptr;
        w.more = u + 1 < U;

        // the memory of this user does not wait for the anchor: the first loads go out before the exchange ends
        float4 ev[CP_AHEAD];
        if (full) {
#pragma unroll
            for (int k = 0; k < CP_AHEAD; ++k)
                ev[k] = k < KPT ? ld_stream_f4(w.eu + k * CP_RUN_STRIDE + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
#pragma unroll
            for (int k = 0; k < CP_AHEAD; ++k)
                ev[k] = k < KPT ? ld4_run(w.eu + k * CP_RUN_STRIDE, w.left - k * CP_RUN_STRIDE, lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }

        const uint32_t mm = coop_collect_max(slots + (int64_t)u * G, G, spin_limit, red, status);
        int A = (int)(mm >> 23) - 127;
        A = A > 127 ? 127 : A;
        A = A < F - 126 ? F - 126 : A;
        if (blockIdx.x == 0 && threadIdx.x == 0) anchor[u] = A;
        w.A = A;
        w.e_min = A - F + 1;

        if (full) coop_convert_user<KPT, HIST, true>(w, gr, ev);
        else coop_convert_user<KPT, HIST, false>(w, gr, ev);

        if (w.more) {
            uint32_t m = 0;
#pragma unroll
            for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
            coop_publish_max(m, slots + (int64_t)(u + 1) * G, red);
        }
        if (HIST) {
            // the workgroup's counts of this user -> global counters: entry j = symbol * copies + replica; a lane
            // adds the eight wavefronts' entry j, the lanes of one symbol (consecutive) are summed by exchange
            __syncthreads();
            for (int j = threadIdx.x; j < K * copies; j += CP_BLOCK) {       // whole wavefronts take part or not
                uint32_t c = 0;
#pragma unroll
                for (int wv = 0; wv < CP_WAVES; ++wv) {
                    c += hist[wv * CP_HIST_SLOTS + j];
                    hist[wv * CP_HIST_SLOTS + j] = 0u;
                }
                for (int o = copies >> 1; o >= 1; o >>= 1) c += (uint32_t)__shfl_xor((int)c, o, CO3_WAVE);
                // (every workgroup adding to the same K words at the same moment serialises chip-wide, and the
                // loads behind the atomics wait: the counts go to one of several partial tables)
                if ((j & (copies - 1)) == 0 && c)
                    atomicAdd(&counts[((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + u) * K + j / copies], c);
            }
            __syncthreads();
        }
    }
}

// Runs per lane that the kernel is built for; a batch takes the smallest one that covers it.
static const int kCoopKpt[] = {1, 2, 4, 8, 12, 16, CP_KPT_MAX};

// Whether the resident-grid form serves this batch on a device with `cus` compute units; *kpt_out and
// *grid_out then hold the launch shape.
bool co3_coop_fits(int64_t n, int cus, int *kpt_out, int *grid_out)
{
    if (cus < 1 || n < 1) return false;
    const int64_t per_wg_step = (int64_t)CP_WAVES * CP_STEP;                       // 2048 elements
    const int64_t need = (n + (int64_t)cus * per_wg_step - 1) / ((int64_t)cus * per_wg_step);
    if (need > CP_KPT_MAX) return false;
    int kpt = CP_KPT_MAX;
    for (int i = (int)(sizeof(kCoopKpt) / sizeof(kCoopKpt[0])) - 1; i >= 0; --i)
        if (kCoopKpt[i] >= need) kpt = kCoopKpt[i];
    const int64_t grid = (n + kpt * per_wg_step - 1) / (kpt * per_wg_step);         // <= cus
    *kpt_out = kpt;
    *grid_out = (int)grid;
    return true;
}

template <int KPT>
static void coop_launch_kpt(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int grid,
                            int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, uint32_t *slots,
                            uint32_t spin_limit, int32_t *status, hipStream_t st)
{
    if (counts)
        hipLaunchKernelGGL((k_coop_convert<KPT, true>), dim3(grid), dim3(CP_BLOCK), 0, st, g, err, sym, n, stride, U, anchor,
                           gamma, fmt, counts, slots, spin_limit, status);
    else
        hipLaunchKernelGGL((k_coop_convert<KPT, false>), dim3(grid), dim3(CP_BLOCK), 0, st, g, err, sym, n, stride, U, anchor,
                           gamma, fmt, counts, slots, spin_limit, status);
}

hipError_t co3_launch_coop_convert(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int kpt,
                                   int grid, int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts,
                                   uint32_t *slots, uint32_t spin_limit, int32_t *status, hipStream_t st)
{
    Co3LaunchTimer tm(CO3_K_COOP, st);
#define CO3_COOP_CASE(KPT)                                                                                         \
    case KPT:                                                                                                      \
        coop_launch_kpt<KPT>(g, err, sym, n, U, stride, grid, anchor, gamma, fmt, counts, slots, spin_limit, status, st); \
        break
    switch (kpt) {
        CO3_COOP_CASE(1);
        CO3_COOP_CASE(2);
        CO3_COOP_CASE(4);
        CO3_COOP_CASE(8);
        CO3_COOP_CASE(12);
        CO3_COOP_CASE(16);
        CO3_COOP_CASE(CP_KPT_MAX);
    default: return hipErrorInvalidValue;
    }
#undef CO3_COOP_CASE
    return hipGetLastError();
}
