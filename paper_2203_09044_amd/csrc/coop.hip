// User side of Algorithm 1 with every gradient read once: the exponent anchor of a user needs the
// largest magnitude of the whole vector before the first element can be converted, so a pass of its
// own over g reads 4 of the path's 16 bytes per element a second time.  Here one resident grid (one
// workgroup of 512 lanes per compute unit) holds a user's whole gradient in registers between the two
// uses: every workgroup owns the same contiguous 1/G of each user's vector, loads its part of g, takes
// the largest magnitude, exchanges it with the other workgroups through one word per workgroup in
// global memory, and converts from registers.  While user u is converted, each register that has been
// consumed is refilled with user u+1's gradient (the last few runs of u+1 have registers of their own and are
// requested first), so the exchange for u+1 starts when u ends.
//
// The exchange uses no fences: a workgroup publishes one self-validating 32-bit word (valid bit |
// magnitude bits) with a relaxed device-scope store, and one wavefront of every workgroup polls the G
// words with relaxed device-scope loads until all are valid.  Nothing else is communicated inside the
// kernel, so no cache needs flushing.  Every wait is bounded: after `spin_limit` polls the workgroup
// raises CO3_ETIMEOUT and goes on with the anchor at its lower clamp (results are then unspecified, but
// in bounds, and the grid drains).
#include "co3_dev.h"
#include "kernels.h"

#include <atomic>

#define CP_BLOCK 512
#define CP_WAVES (CP_BLOCK / CO3_WAVE)
#define CP_VEC 4
#define CP_STEP (CO3_WAVE * CP_VEC)          // elements that one load of a wavefront covers: one KiB
#define CP_KPT_MAX CO3_COOP_KPT_MAX          // steps per lane: 16-byte pieces of g that a lane keeps in registers
#define CP_KPT_REG_MAX 32                    // the most that the all-register form is built for
#ifndef CP_AHEAD
#define CP_AHEAD 6                           // memory loads in flight per lane ahead of the conversion
#endif
#ifndef CP_SPARE
#define CP_SPARE 4                           // runs of the next user's gradient that have registers of their own
#endif
#define CP_HIST_SLOTS 1024                   // LDS counters per wavefront
// Registers: a workgroup brings two wavefronts per SIMD, and the kernel is compiled for that (191 vector
// registers with CP_SPARE 4).  While it runs, a kernel of another stream finds little room beside it; with 3 the
// kernel keeps to 168 registers and needs CP_SPARE 1 to stay free of spills (5 us slower on 10 users x 11M).
#ifndef CP_WAVES_PER_SIMD
#define CP_WAVES_PER_SIMD 2
#endif
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

// One user's conversion by one wavefront whose KPT runs of 256 elements all lie below n: the gradient from
// registers, the memory streamed CP_AHEAD runs ahead; as soon as a run is converted its registers take the
// next user's gradient.  Straight-line code: the compiler can count the memory operations in flight exactly.
struct CoopWave {
    float *eu;                 // the user's memory there
    uint8_t *su;               // its symbols there
    const float *gnext;        // the next user's gradient there (read when `more`)
    bool more;
    int64_t left;              // n - (first element of the wavefront's run 0)
    uint32_t lane4;
    int A, e_min, E, M, codemax;
    float gamma;
    uint32_t *myhist;
    int copies, mycopy;
};

// Run k of the wavefront (gradient gv, memory e4): conversion, new memory and symbols out, counts.
template <bool NIB>
__device__ __forceinline__ void coop_convert_run(const CoopWave &w, int k, const float4 gv, const float4 e4)
{
    const float ga[CP_VEC] = {gv.x, gv.y, gv.z, gv.w}, ea[CP_VEC] = {e4.x, e4.y, e4.z, e4.w};
    float en[CP_VEC];
    uint32_t q[CP_VEC];
#pragma unroll
    for (int c = 0; c < CP_VEC; ++c) {
        const float x = ga[c] + w.gamma * ea[c];              // no contraction (build flag): one rounding per operation
        float v;
        co3_quantize(x, w.e_min, w.A, w.E, w.M, w.codemax, q[c], v);
        en[c] = x - v;
    }
    st_stream_f4(w.eu + k * CP_STEP + w.lane4, make_float4(en[0], en[1], en[2], en[3]));
    if (NIB)         // two symbols per byte, the earlier one in the low half
        *reinterpret_cast<uint16_t *>(w.su + k * (CP_STEP / 2) + w.lane4 / 2) =
            (uint16_t)(q[0] | (q[1] << 4) | (q[2] << 8) | (q[3] << 12));
    else
        *reinterpret_cast<uint32_t *>(w.su + k * CP_STEP + w.lane4) = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
#pragma unroll
    for (int c = 0; c < CP_VEC; ++c) atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
}

// The same with an anchor per element (a4: the four anchors of the lane's elements, a byte each).
template <bool NIB>
__device__ __forceinline__ void coop_convert_run_a4(const CoopWave &w, int k, const float4 gv, const float4 e4, uint32_t a4,
                                                    int F)
{
    const float ga[CP_VEC] = {gv.x, gv.y, gv.z, gv.w}, ea[CP_VEC] = {e4.x, e4.y, e4.z, e4.w};
    float en[CP_VEC];
    uint32_t q[CP_VEC];
#pragma unroll
    for (int c = 0; c < CP_VEC; ++c) {
        const int A = (int)(int8_t)(a4 >> (8 * c));
        const float x = ga[c] + w.gamma * ea[c];
        float v;
        co3_quantize(x, A - F + 1, A, w.E, w.M, w.codemax, q[c], v);
        en[c] = x - v;
    }
    st_stream_f4(w.eu + k * CP_STEP + w.lane4, make_float4(en[0], en[1], en[2], en[3]));
    if (NIB)
        *reinterpret_cast<uint16_t *>(w.su + k * (CP_STEP / 2) + w.lane4 / 2) =
            (uint16_t)(q[0] | (q[1] << 4) | (q[2] << 8) | (q[3] << 12));
    else
        *reinterpret_cast<uint32_t *>(w.su + k * CP_STEP + w.lane4) = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
#pragma unroll
    for (int c = 0; c < CP_VEC; ++c) atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
}

template <int KPT, bool NIB>
__device__ __forceinline__ void coop_convert_user(const CoopWave &w, float4 (&gr)[KPT], float4 (&ev)[CP_AHEAD],
                                                  float4 (&sp)[CP_SPARE])
{
    constexpr int S = KPT > CP_SPARE ? CP_SPARE : 0;     // the next user's last S runs were requested before this call
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        float *ek = w.eu + k * CP_STEP;
        const float4 gv = gr[k], e4 = ev[k % CP_AHEAD];
        if (k + CP_AHEAD < KPT) ev[k % CP_AHEAD] = ld_stream_f4(ek + CP_AHEAD * CP_STEP + w.lane4);
        coop_convert_run<NIB>(w, k, gv, e4);
        // the registers are free: the next user's gradient moves in
        if (k >= KPT - S)
            gr[k] = sp[k - (KPT - S)];
        else if (w.more)
            gr[k] = ld_stream_f4(w.gnext + k * CP_STEP + w.lane4);
    }
}

// The one wavefront that holds the ragged end of the vector (fewer than KPT whole runs) and those after it,
// which hold nothing, only take part in the search for the largest magnitude, run by run with every access
// guarded; the ragged end is converted after the kernel by the plain conversion kernel, with the anchors
// that this kernel leaves.  (A guarded copy of the conversion in here would add its registers to those of
// the path above, which every other wavefront of the device runs.)
__device__ __forceinline__ uint32_t coop_ragged_max(const float *gu, int64_t left, int kpt, uint32_t lane4)
{
    uint32_t m = 0;
#pragma unroll 1
    for (int k = 0; k < kpt; ++k) {
        const int64_t rem = left - (int64_t)k * CP_STEP;
        if (rem <= 0) break;
        m = absbits4(ld4_run(gu + k * CP_STEP, rem, lane4), m);
    }
    return m;
}

// The symbol counts of the user just converted.  Entry j of a wavefront's counters = symbol * copies + replica.
// Every wavefront adds up its own counters: a lane takes consecutive entries (all of one symbol, or whole
// symbols), lanes that share a symbol finish by exchange.  The wavefronts' sums are added up and go to one of
// several partial tables (every workgroup adding to the same K words at the same moment serialises chip-wide,
// and the loads behind the atomics wait).  Called by all threads of the workgroup; the counters are zero
// afterwards.  (`wavecnt` is not written again before the barriers of the next exchange.)
__device__ __forceinline__ void coop_flush_counts(uint32_t *hist, uint32_t *wavecnt, int wave, int lane, int K, int copies,
                                                  uint32_t *__restrict__ counts_row)
{
    const int per = K * copies / CO3_WAVE;                 // entries per lane: a power of two, 2 .. 16
    const int grp = per < copies ? per : copies;           // entries of one symbol that a lane holds together
    uint32_t *h = hist + wave * CP_HIST_SLOTS;
    for (int c0 = 0; c0 < per; c0 += grp) {
        const int base = lane * per + c0;
        uint32_t sum = 0;
        for (int i = 0; i < grp; ++i) {
            sum += h[base + i];
            h[base + i] = 0u;
        }
        for (int o = 1; o * grp < copies; o <<= 1) sum += (uint32_t)__shfl_xor((int)sum, o, CO3_WAVE);
        if (base % copies == 0) wavecnt[wave * 256 + base / copies] = sum;
    }
    __syncthreads();
    if ((int)threadIdx.x < K) {
        uint32_t c = 0;
#pragma unroll
        for (int wv = 0; wv < CP_WAVES; ++wv) c += wavecnt[wv * 256 + threadIdx.x];
        if (c) atomicAdd(&counts_row[threadIdx.x], c);
    }
}

#ifdef CO3_COOP_TRACE
__device__ unsigned long long co3_coop_trace[4 * 64 * 8];
#define CP_TRACE(i)                                                                                   \
    if (threadIdx.x == 0 && (blockIdx.x & 63) == 0 && u < 64)                                         \
        co3_coop_trace[((blockIdx.x >> 6) * 64 + u) * 8 + (i)] = wall_clock64();
extern "C" int co3_debug_coop_trace(unsigned long long *host)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(co3_coop_trace), sizeof(co3_coop_trace));
}
#else
#define CP_TRACE(i)
#endif

// grid: G workgroups (at most one per compute unit, all resident); workgroup w owns elements
// [w * KPT * 2048, (w + 1) * KPT * 2048) of every user, wavefront v of it the v-th eighth, lane l of the
// wavefront elements 4l .. 4l+3 of each of the wavefront's KPT runs of 256.
template <int KPT, bool NIB>
__global__ __launch_bounds__(CP_BLOCK) __attribute__((amdgpu_waves_per_eu(CP_WAVES_PER_SIMD, CP_WAVES_PER_SIMD))) void k_coop_convert(const float *__restrict__ g, float *__restrict__ err,
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
    __shared__ uint32_t hist[CP_WAVES * CP_HIST_SLOTS];
    __shared__ uint32_t wavecnt[CP_WAVES * 256];               // symbol counts of every wavefront's part of a user
    const int copies = CP_HIST_SLOTS / K > 32 ? 32 : CP_HIST_SLOTS / K;
    for (int j = threadIdx.x; j < CP_WAVES * CP_HIST_SLOTS; j += CP_BLOCK) hist[j] = 0u;

    // first element of the wavefront's run 0 (uniform); run k lies k * CP_STEP further
    const int64_t first = (((int64_t)blockIdx.x * CP_WAVES + wave) * KPT) * CP_STEP;
    const uint32_t lane4 = (uint32_t)lane * CP_VEC;
    const bool full = first + (int64_t)KPT * CP_STEP <= n;      // uniform: every run of the wavefront is whole

    // user 0's gradient: every load of the lane in flight at once
    float4 gr[KPT];
    {
        uint32_t m = 0;
        if (full) {
#pragma unroll
            for (int k = 0; k < KPT; ++k) gr[k] = ld_stream_f4(g + first + k * CP_STEP + lane4);
#pragma unroll
            for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
        } else {
#pragma unroll
            for (int k = 0; k < KPT; ++k) gr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            m = coop_ragged_max(g + first, n - first, KPT, lane4);
        }
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
        w.su = NIB ? sym + (int64_t)u * (stride / 2) + first / 2 : sym + (int64_t)u * stride + first;
        w.more = u + 1 < U;

        // the memory of this user does not wait for the anchor: the first loads go out before the exchange ends
        float4 ev[CP_AHEAD];
        CP_TRACE(0)
#pragma unroll
        for (int k = 0; k < CP_AHEAD; ++k)
            ev[k] = full && k < KPT ? ld_stream_f4(w.eu + k * CP_STEP + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);

        // the next user's last runs have registers of their own and are requested now: when this user's
        // conversion ends, all of the next user's gradient has been on its way for CP_SPARE runs' time
        constexpr int S = KPT > CP_SPARE ? CP_SPARE : 0;
        float4 sp[CP_SPARE];
#pragma unroll
        for (int i = 0; i < CP_SPARE; ++i)
            sp[i] = (i < S && full && w.more) ? ld_stream_f4(w.gnext + (KPT - S + i) * CP_STEP + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);

        // the counts of the user before this one leave the workgroup while the exchange is on its way
        if (u > 0) coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + u - 1) * K);
        CP_TRACE(5)
        const uint32_t mm = coop_collect_max(slots + (int64_t)u * G, G, spin_limit, red, status);
        int A = (int)(mm >> 23) - 127;
        A = A > 127 ? 127 : A;
        A = A < F - 126 ? F - 126 : A;
        if (blockIdx.x == 0 && threadIdx.x == 0) anchor[u] = A;
        w.A = A;
        w.e_min = A - F + 1;
        CP_TRACE(1)

        if (full) coop_convert_user<KPT, NIB>(w, gr, ev, sp);
        CP_TRACE(2)

        if (w.more) {
            uint32_t m = 0;
            if (full) {
#pragma unroll
                for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
            } else {
                m = coop_ragged_max(w.gnext, w.left, KPT, lane4);
            }
#ifdef CO3_COOP_TRACE
            asm volatile("" ::"v"(m));                // the time stamp comes after the loads have landed
#endif
            CP_TRACE(3)
            coop_publish_max(m, slots + (int64_t)(u + 1) * G, red);
            CP_TRACE(4)
        }
    }
    coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + U - 1) * K);
}

// ---- several tensors per user: one anchor per (user, tensor) ------------------------------------------
// The same resident grid when a user's vector is a concatenation of tensors, each with its own anchor.  The
// workgroups do not exchange one maximum but add their tensors' maxima into a table [U][nseg] in global memory
// (device-scope atomic max, the returned values awaited), then publish a word that only says "done"; a
// workgroup that has seen every word reads the maxima of the tensors it holds.  A run of 256 elements that
// lies in one tensor is converted from registers with that tensor's anchor; the few runs that hold a tensor
// boundary are converted after the others, element by element, from memory.
__device__ __forceinline__ void wave_lds_sync_coop() { co3_wave_lds_sync(); }

#define CP_SEGS_STASH 3                      // runs with a tensor boundary per wavefront that wait in LDS (more: read again)
#define CP_SEGS_LDS_BYTES(KPT) (CP_WAVES * CP_SEGS_STASH * CP_STEP * 4 + CP_WAVES * (KPT) * CO3_WAVE * 4)

__device__ __forceinline__ void coop_max_agent(uint32_t *p, uint32_t v)
{
    (void)__hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int coop_anchor_of(uint32_t maxbits, int F)
{
    int A = (int)(maxbits >> 23) - 127;
    A = A > 127 ? 127 : A;
    return A < F - 126 ? F - 126 : A;
}

// Tensor of element e, searched upwards from tensor s (which starts at or before e).
__device__ __forceinline__ int coop_seg_from(const int64_t *seg_off, int nseg, int s, int64_t e)
{
    while (s + 1 < nseg && seg_off[s + 1] <= e) ++s;
    return s;
}

// Maxima found by a wavefront wait in its lanes (entry i in lane i) and go out together, one atomic each: an
// atomic that is waited for costs a trip to memory, and the waits the compiler puts at the end of a loop body
// would line these trips up one after the other.
struct CoopPending {
    int count;          // uniform
    int seg;            // lane i: tensor of entry i
    uint32_t max;
};
__device__ __forceinline__ void coop_pending_flush(CoopPending &p, uint32_t *tmax_u)
{
    if ((int)(threadIdx.x & (CO3_WAVE - 1)) < p.count && p.max) coop_max_agent(tmax_u + p.seg, p.max);
    p.count = 0;
}
__device__ __forceinline__ void coop_pending_add(CoopPending &p, int seg, uint32_t m, uint32_t *tmax_u)
{
    if ((int)(threadIdx.x & (CO3_WAVE - 1)) == p.count) {
        p.seg = seg;
        p.max = m;
    }
    if (++p.count == CO3_WAVE) coop_pending_flush(p, tmax_u);
}

// Maxima of a run of 256 elements that holds tensor boundaries: tensor by tensor (a uniform loop over the
// tensors that the run touches), the wavefront's maximum over the tensor's elements as one entry.  v: the
// lane's four elements from element e_run + 4 * lane on; s_first: the tensor of element e_run.
__device__ __forceinline__ void coop_segmax_run(const float4 v, int64_t e_run, uint32_t lane4, int64_t n, const int64_t *seg_off,
                                                int nseg, int s_first, uint32_t *tmax_u, CoopPending &pend)
{
    const uint32_t bits[4] = {__float_as_uint(v.x) & 0x7fffffffu, __float_as_uint(v.y) & 0x7fffffffu,
                              __float_as_uint(v.z) & 0x7fffffffu, __float_as_uint(v.w) & 0x7fffffffu};
    const int64_t end = e_run + CP_STEP < n ? e_run + CP_STEP : n;      // uniform
    const int64_t e = e_run + lane4;
    for (int sg = s_first; sg < nseg; ++sg) {                               // uniform
        const int64_t a = seg_off[sg], b = seg_off[sg + 1];
        if (a >= end) break;
        uint32_t m = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (e + c >= a && e + c < b && e + c < end) m = m > bits[c] ? m : bits[c];
        m = wave_max_u32(m);
        coop_pending_add(pend, sg, m, tmax_u);
    }
}

template <int KPT, bool NIB>
__global__ __launch_bounds__(CP_BLOCK) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_coop_convert_segs(
    const float *__restrict__ g, float *__restrict__ err, uint8_t *__restrict__ sym, int64_t n, int64_t stride, int U,
    const int64_t *__restrict__ seg_off_g, int nseg, int32_t *__restrict__ anchor, float gamma, co3_fmt fmt,
    uint32_t *__restrict__ counts, uint32_t *__restrict__ slots, uint32_t *__restrict__ tmax, uint32_t spin_limit,
    int32_t *status)
{
    const FmtC fc(fmt);
    const int F = fc.F, K = fc.K;
    const int G = gridDim.x;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / CO3_WAVE);
    __shared__ uint32_t red[CP_WAVES + 1];
    __shared__ uint32_t hist[CP_WAVES * CP_HIST_SLOTS];
    __shared__ uint32_t wavecnt[CP_WAVES * 256];
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    const int copies = CP_HIST_SLOTS / K > 32 ? 32 : CP_HIST_SLOTS / K;
    for (int j = threadIdx.x; j < CP_WAVES * CP_HIST_SLOTS; j += CP_BLOCK) hist[j] = 0u;
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);     // (the launch keeps nseg + 1 within the cache)

    const int64_t first = (((int64_t)blockIdx.x * CP_WAVES + wave) * KPT) * CP_STEP;
    const uint32_t lane4 = (uint32_t)lane * CP_VEC;
    const bool full = first + (int64_t)KPT * CP_STEP <= n;

    // Tensor of every run's first element (lane k looks run k up; kept in LDS, read where a run needs it), and
    // as bit masks over the runs: which hold a tensor boundary, which start in another tensor than the run
    // before, after which the maximum gathered so far belongs to a tensor that ends.  The same for every user.
    static_assert(KPT <= 32, "a lane per run, masks of 64 bits");
    __shared__ int segs_s[CP_WAVES][32];
    __shared__ int8_t anchor_s[CO3_SEG_CACHE];             // the current user's anchor of every tensor
    __shared__ uint8_t runa_s[CP_WAVES][32];                // ... of the tensor of every run's first element
    // runs with a tensor boundary wait here (gradient, memory) between the pass over all runs and their own loop
    extern __shared__ __align__(16) unsigned char coop_segs_lds[];
    float4 *stash_g = reinterpret_cast<float4 *>(coop_segs_lds);
    // the anchors of the current user for every (run, lane): four bytes, one per element
    uint32_t *a4_s = reinterpret_cast<uint32_t *>(stash_g + CP_WAVES * CP_SEGS_STASH * CO3_WAVE) + (size_t)wave * KPT * CO3_WAVE;
    uint64_t strad, newm, flushm;
    {
        const int64_t e0 = first + (int64_t)lane * CP_STEP;
        const bool have = lane < KPT && e0 < n;
        const int sk = have ? co3_find_seg(seg_off, nseg, e0) : nseg - 1;
        const int64_t last = e0 + CP_STEP - 1 < n ? e0 + CP_STEP - 1 : n - 1;
        const bool st = have && co3_find_seg(seg_off, nseg, last) != sk;
        if (lane < 32) segs_s[wave][lane] = sk;
        const int prev = __shfl_up(sk, 1, CO3_WAVE);
        strad = __ballot(st);
        newm = __ballot(lane < KPT && (lane == 0 || prev != sk));
        flushm = ((strad | newm) >> 1) | (1ull << (KPT - 1));
        wave_lds_sync_coop();
    }

    // maxima of the user whose gradient the registers hold -> tmax[uu]; returns what must be awaited
    float4 gr[KPT];
    auto seg_maxima = [&](int uu, const float *gu) {
        uint32_t *tm = tmax + (int64_t)uu * nseg;
        CoopPending pend = {0, 0, 0u};
        if (full) {
            uint32_t acc = 0;
            int held = 0;                                // uniform: runs with a tensor boundary met so far
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                if ((strad >> k) & 1ull) {               // uniform: set aside for the loop below
                    if (held < CP_SEGS_STASH) stash_g[(wave * CP_SEGS_STASH + held) * CO3_WAVE + lane] = gr[k];
                    ++held;
                } else {
                    acc = absbits4(gr[k], acc);
                    if ((flushm >> k) & 1ull) {          // uniform: a tensor's last whole run here
                        coop_pending_add(pend, segs_s[wave][k], wave_max_u32(acc), tm);
                        acc = 0;
                    }
                }
            }
            if (strad) {                                 // uniform: the runs with a tensor boundary, element by element
                int i = 0;
#pragma unroll 1
                for (int k = 0; k < KPT; ++k) {
                    if (!((strad >> k) & 1ull)) continue;
                    const int64_t e0 = first + (int64_t)k * CP_STEP;
                    const float4 v = i < CP_SEGS_STASH ? stash_g[(wave * CP_SEGS_STASH + i) * CO3_WAVE + lane]
                                                       : ld_stream_f4(gu + e0 + lane4);
                    coop_segmax_run(v, e0, lane4, n, seg_off, nseg, segs_s[wave][k], tm, pend);
                    ++i;
                }
            }
        } else {                                         // the ragged end, or nothing
#pragma unroll 1
            for (int k = 0; k < KPT; ++k) {
                const int64_t e0 = first + (int64_t)k * CP_STEP;
                if (e0 >= n) break;
                const float4 v = ld4_run(gu + e0, n - e0, lane4);
                coop_segmax_run(v, e0, lane4, n, seg_off, nseg, co3_find_seg(seg_off, nseg, e0), tm, pend);
            }
        }
        coop_pending_flush(pend, tm);
    };
    // "done" of this workgroup for a user: after every wavefront's atomics have returned
    auto publish_done = [&](uint32_t *row) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // this wavefront's atomics have been performed
        __syncthreads();
        if (threadIdx.x == 0) st_relaxed_agent(row + blockIdx.x, CP_VALID);
    };

    {
        if (full) {
#pragma unroll
            for (int k = 0; k < KPT; ++k) gr[k] = ld_stream_f4(g + first + k * CP_STEP + lane4);
        } else {
#pragma unroll
            for (int k = 0; k < KPT; ++k) gr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        seg_maxima(0, g);
        publish_done(slots);
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
        w.gnext = g + (int64_t)(u + 1) * stride + first;
        w.eu = err + (int64_t)u * stride + first;
        w.su = NIB ? sym + (int64_t)u * (stride / 2) + first / 2 : sym + (int64_t)u * stride + first;
        w.more = u + 1 < U;
        const uint32_t *tm = tmax + (int64_t)u * nseg;

        float4 ev[CP_AHEAD];
        CP_TRACE(0)
#pragma unroll
        for (int k = 0; k < CP_AHEAD; ++k)
            ev[k] = full && k < KPT ? ld_stream_f4(w.eu + k * CP_STEP + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (u > 0) coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + u - 1) * K);
        (void)coop_collect_max(slots + (int64_t)u * G, G, spin_limit, red, status);    // every workgroup's maxima are in
        CP_TRACE(1)

        // anchors: of the tensors of this wavefront's runs, and (workgroup 0) of all tensors for the caller
        for (int s = threadIdx.x; s < nseg; s += CP_BLOCK) {       // (nseg is within the cache: at most one round)
            const int A = coop_anchor_of(ld_relaxed_agent(tm + s), F);
            anchor_s[s] = (int8_t)A;
            if (blockIdx.x == 0) anchor[(int64_t)u * nseg + s] = A;
        }
        __syncthreads();                                 // (read until this user's conversion ends; the next write
                                                         // comes after the barriers of the next exchange)
        CP_TRACE(2)

        if (full) {
            // anchors: a run inside one tensor takes that tensor's anchor for all its elements, a run with a tensor
            // boundary an anchor per element (per lane in LDS); the conversion below is then the same for all
            if (lane < KPT) runa_s[wave][lane] = (uint8_t)anchor_s[segs_s[wave][lane]];      // lane k: run k
            wave_lds_sync_coop();
            if (strad) {                                 // uniform
#pragma unroll 1
                for (int k = 0; k < KPT; ++k) {
                    if (!((strad >> k) & 1ull)) continue;
                    const int64_t e0 = first + (int64_t)k * CP_STEP + lane4;
                    int sg = segs_s[wave][k];
                    uint32_t a4 = 0;
#pragma unroll
                    for (int c = 0; c < CP_VEC; ++c) {
                        sg = coop_seg_from(seg_off, nseg, sg, e0 + c);
                        a4 |= (uint32_t)(uint8_t)anchor_s[sg] << (8 * c);
                    }
                    a4_s[k * CO3_WAVE + lane] = a4;
                }
            }
            wave_lds_sync_coop();
            CP_TRACE(3)
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const float4 gv = gr[k], e4 = ev[k % CP_AHEAD];
                if (k + CP_AHEAD < KPT) ev[k % CP_AHEAD] = ld_stream_f4(w.eu + (k + CP_AHEAD) * CP_STEP + lane4);
                // (both are read; which one counts is the same for the whole wavefront)
                const uint32_t a4 = (strad >> k) & 1ull ? a4_s[k * CO3_WAVE + lane] : (uint32_t)runa_s[wave][k] * 0x01010101u;
                coop_convert_run_a4<NIB>(w, k, gv, e4, a4, F);
                if (w.more) gr[k] = ld_stream_f4(w.gnext + k * CP_STEP + lane4);
            }
        }
        CP_TRACE(4)
        if (w.more) {
            seg_maxima(u + 1, g + (int64_t)(u + 1) * stride);
            CP_TRACE(5)
            publish_done(slots + (int64_t)(u + 1) * G);
            CP_TRACE(6)
        }
    }
    coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + U - 1) * K);
}

// ---- vectors beyond what the registers hold: part of a wavefront's runs in LDS ------------------------
// The same kernel for up to CP_BIG_KPT runs per lane: the first CP_BIG_KL runs of a wavefront wait in LDS
// (one KiB per run and wavefront), the other CP_BIG_KR in registers.  A user's conversion takes the LDS runs
// first; the next user's gradient for an LDS run is requested into one of CP_BIG_D registers when the run has
// been converted and moves to LDS that many runs later.
#define CP_BIG_KR 34
#define CP_BIG_KL 14                         // at most; the kernel is also built for CP_BIG_KL_SMALL
#define CP_BIG_KL_SMALL 6
#define CP_BIG_KPT (CP_BIG_KR + CP_BIG_KL)
#define CP_BIG_KPT_SMALL (CP_BIG_KR + CP_BIG_KL_SMALL)
#ifndef CP_BIG_AHEAD
#define CP_BIG_AHEAD 4
#endif
#ifndef CP_BIG_D
#define CP_BIG_D 4
#endif
#define CP_BIG_LDS_BYTES(KL) (CP_WAVES * (KL) * CP_STEP * 4)
static_assert(CP_BIG_KR >= CP_BIG_D && CP_BIG_KL_SMALL >= CP_BIG_D, "the last LDS runs of the next user move in during the register runs");
static_assert(CP_BIG_KPT == CO3_COOP_KPT_BIG, "runs per lane of the large form");

// Returns the largest magnitude pattern of the next user's LDS runs (0 without a next user).
template <int KL, bool NIB>
__device__ __forceinline__ uint32_t coop_convert_user_big(const CoopWave &w, float4 (&gr)[CP_BIG_KR], float4 (&ev)[CP_BIG_AHEAD],
                                                          float4 *lg, int lane)
{
    constexpr int KR = CP_BIG_KR, KPT = KR + KL, A = CP_BIG_AHEAD, D = CP_BIG_D;
    float4 tmp[D];
#pragma unroll
    for (int d = 0; d < D; ++d) tmp[d] = make_float4(0.f, 0.f, 0.f, 0.f);
    uint32_t mnext = 0;
    float4 gl = lg[lane];                       // LDS run 0
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        const float4 e4 = ev[k % A];
        if (k + A < KPT) ev[k % A] = ld_stream_f4(w.eu + (k + A) * CP_STEP + w.lane4);
        float4 gv;
        if (k < KL) {
            gv = gl;
            if (k + 1 < KL) gl = lg[(k + 1) * CO3_WAVE + lane];
        } else
            gv = gr[k - KL];
        coop_convert_run<NIB>(w, k, gv, e4);
        if (w.more) {
            if (k >= D && k - D < KL) {         // the request of D runs ago has had its time: to LDS
                mnext = absbits4(tmp[(k - D) % D], mnext);
                lg[(k - D) * CO3_WAVE + lane] = tmp[(k - D) % D];
            }
            if (k < KL)
                tmp[k % D] = ld_stream_f4(w.gnext + k * CP_STEP + w.lane4);
            else
                gr[k - KL] = ld_stream_f4(w.gnext + k * CP_STEP + w.lane4);
        }
    }
    return mnext;
}

template <int KL, bool NIB>
__global__ __launch_bounds__(CP_BLOCK) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_coop_convert_big(
    const float *__restrict__ g, float *__restrict__ err, uint8_t *__restrict__ sym, int64_t n, int64_t stride, int U,
    int32_t *__restrict__ anchor, float gamma, co3_fmt fmt, uint32_t *__restrict__ counts, uint32_t *__restrict__ slots,
    uint32_t spin_limit, int32_t *status)
{
    constexpr int KR = CP_BIG_KR, KPT = KR + KL;
    const FmtC fc(fmt);
    const int F = fc.F, K = fc.K;
    const int G = gridDim.x;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / CO3_WAVE);
    __shared__ uint32_t red[CP_WAVES + 1];
    __shared__ uint32_t hist[CP_WAVES * CP_HIST_SLOTS];
    __shared__ uint32_t wavecnt[CP_WAVES * 256];
    extern __shared__ __align__(16) unsigned char coop_big_lds[];
    float4 *lg = reinterpret_cast<float4 *>(coop_big_lds) + (size_t)wave * KL * CO3_WAVE;   // the wavefront's LDS runs
    const int copies = CP_HIST_SLOTS / K > 32 ? 32 : CP_HIST_SLOTS / K;
    for (int j = threadIdx.x; j < CP_WAVES * CP_HIST_SLOTS; j += CP_BLOCK) hist[j] = 0u;

    const int64_t first = (((int64_t)blockIdx.x * CP_WAVES + wave) * KPT) * CP_STEP;
    const uint32_t lane4 = (uint32_t)lane * CP_VEC;
    const bool full = first + (int64_t)KPT * CP_STEP <= n;

    // user 0: the LDS runs pass through the registers of the register runs
    float4 gr[KR];
    {
        uint32_t m = 0;
        if (full) {
#pragma unroll
            for (int k = 0; k < KL; ++k) gr[k] = ld_stream_f4(g + first + k * CP_STEP + lane4);
#pragma unroll
            for (int k = 0; k < KL; ++k) {
                m = absbits4(gr[k], m);
                lg[k * CO3_WAVE + lane] = gr[k];
            }
#pragma unroll
            for (int k = 0; k < KR; ++k) gr[k] = ld_stream_f4(g + first + (KL + k) * CP_STEP + lane4);
#pragma unroll
            for (int k = 0; k < KR; ++k) m = absbits4(gr[k], m);
        } else {
#pragma unroll
            for (int k = 0; k < KR; ++k) gr[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            m = coop_ragged_max(g + first, n - first, KPT, lane4);
        }
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
        w.gnext = g + (int64_t)(u + 1) * stride + first;
        w.eu = err + (int64_t)u * stride + first;
        w.su = NIB ? sym + (int64_t)u * (stride / 2) + first / 2 : sym + (int64_t)u * stride + first;
        w.more = u + 1 < U;

        float4 ev[CP_BIG_AHEAD];
#pragma unroll
        for (int k = 0; k < CP_BIG_AHEAD; ++k)
            ev[k] = full ? ld_stream_f4(w.eu + k * CP_STEP + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (u > 0) coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + u - 1) * K);
        const uint32_t mm = coop_collect_max(slots + (int64_t)u * G, G, spin_limit, red, status);
        int A = (int)(mm >> 23) - 127;
        A = A > 127 ? 127 : A;
        A = A < F - 126 ? F - 126 : A;
        if (blockIdx.x == 0 && threadIdx.x == 0) anchor[u] = A;
        w.A = A;
        w.e_min = A - F + 1;

        uint32_t m = 0;
        if (full) m = coop_convert_user_big<KL, NIB>(w, gr, ev, lg, lane);
        if (w.more) {
            if (full) {
#pragma unroll
                for (int k = 0; k < KR; ++k) m = absbits4(gr[k], m);
            } else {
                m = coop_ragged_max(w.gnext, w.left, KPT, lane4);
            }
            coop_publish_max(m, slots + (int64_t)(u + 1) * G, red);
        }
    }
    coop_flush_counts(hist, wavecnt, wave, lane, K, copies, counts + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + U - 1) * K);
}

// Runs per lane that the kernel is built for; a batch takes the smallest one that covers it.
static const int kCoopKpt[] = {1, 2, 4, 8, 12, 16, CP_KPT_MAX, CP_KPT_REG_MAX, CP_BIG_KPT_SMALL, CP_BIG_KPT};

// Whether the resident-grid form serves this batch on a device with `cus` compute units; *kpt_out and
// *grid_out then hold the launch shape.
// (the form for several tensors per user is built for fewer sizes)
static const int kCoopKptSegs[] = {1, 4, 12, CP_KPT_MAX, CP_KPT_REG_MAX};

bool co3_coop_fits(int64_t n, int nseg, int cus, int *kpt_out, int *grid_out)
{
    if (nseg > 1) {
        if (cus < 1 || n < 1 || nseg + 1 > CO3_SEG_CACHE) return false;
        const int64_t step = (int64_t)CP_WAVES * CP_STEP;
        const int64_t need = (n + (int64_t)cus * step - 1) / ((int64_t)cus * step);
        if (need > CP_KPT_REG_MAX) return false;
        int kpt = CP_KPT_REG_MAX;
        for (int i = (int)(sizeof(kCoopKptSegs) / sizeof(kCoopKptSegs[0])) - 1; i >= 0; --i)
            if (kCoopKptSegs[i] >= need) kpt = kCoopKptSegs[i];
        *kpt_out = kpt;
        *grid_out = (int)((n + kpt * step - 1) / (kpt * step));
        return true;
    }
    if (cus < 1 || n < 1) return false;
    const int64_t per_wg_step = (int64_t)CP_WAVES * CP_STEP;                       // 2048 elements
    const int64_t need = (n + (int64_t)cus * per_wg_step - 1) / ((int64_t)cus * per_wg_step);
    if (need > CP_BIG_KPT) return false;
    int kpt = CP_BIG_KPT;
    for (int i = (int)(sizeof(kCoopKpt) / sizeof(kCoopKpt[0])) - 1; i >= 0; --i)
        if (kCoopKpt[i] >= need) kpt = kCoopKpt[i];
    const int64_t grid = (n + kpt * per_wg_step - 1) / (kpt * per_wg_step);         // <= cus
    *kpt_out = kpt;
    *grid_out = (int)grid;
    return true;
}

int64_t co3_coop_full_elements(int64_t n, int kpt)
{
    const int64_t part = (int64_t)kpt * CP_STEP;
    return n / part * part;
}


template <int KPT>
static void coop_launch_kpt(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int grid,
                            int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, uint32_t *slots,
                            uint32_t spin_limit, int32_t *status, int sym_nib, hipStream_t st)
{
    if (sym_nib)
        hipLaunchKernelGGL((k_coop_convert<KPT, true>), dim3(grid), dim3(CP_BLOCK), 0, st, g, err, sym, n, stride, U, anchor,
                           gamma, fmt, counts, slots, spin_limit, status);
    else
        hipLaunchKernelGGL((k_coop_convert<KPT, false>), dim3(grid), dim3(CP_BLOCK), 0, st, g, err, sym, n, stride, U, anchor,
                           gamma, fmt, counts, slots, spin_limit, status);
}

// A kernel that wants more LDS than it gets without asking: asked for once per device (the flag array is the
// caller's, one per kernel).
#define CP_MAX_DEVICES 64
static hipError_t coop_allow_lds(const void *kernel, int bytes, std::atomic<int> (&asked)[CP_MAX_DEVICES])
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= CP_MAX_DEVICES) return hipErrorInvalidDevice;
    if (asked[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) asked[dev].store(1, std::memory_order_release);
    return e;
}

// The form with KL runs per wavefront in LDS.
template <int KL>
static hipError_t coop_launch_big(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int grid,
                                  int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, uint32_t *slots,
                                  uint32_t spin_limit, int32_t *status, int sym_nib, hipStream_t st)
{
    static std::atomic<int> asked[2][CP_MAX_DEVICES];     // zero-initialised
    const void *kernel = sym_nib ? reinterpret_cast<const void *>(k_coop_convert_big<KL, true>)
                                 : reinterpret_cast<const void *>(k_coop_convert_big<KL, false>);
    const hipError_t e = coop_allow_lds(kernel, CP_BIG_LDS_BYTES(KL), asked[sym_nib ? 1 : 0]);
    if (e != hipSuccess) return e;
    if (sym_nib)
        hipLaunchKernelGGL((k_coop_convert_big<KL, true>), dim3(grid), dim3(CP_BLOCK), CP_BIG_LDS_BYTES(KL), st, g, err, sym, n,
                           stride, U, anchor, gamma, fmt, counts, slots, spin_limit, status);
    else
        hipLaunchKernelGGL((k_coop_convert_big<KL, false>), dim3(grid), dim3(CP_BLOCK), CP_BIG_LDS_BYTES(KL), st, g, err, sym, n,
                           stride, U, anchor, gamma, fmt, counts, slots, spin_limit, status);
    return hipGetLastError();
}

template <int KPT>
static hipError_t coop_launch_segs(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int grid,
                             const int64_t *seg_off, int nseg, int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts,
                             uint32_t *slots, uint32_t *tmax, uint32_t spin_limit, int32_t *status, int sym_nib, hipStream_t st)
{
    static std::atomic<int> asked[2][CP_MAX_DEVICES];     // zero-initialised
    const void *kernel = sym_nib ? reinterpret_cast<const void *>(k_coop_convert_segs<KPT, true>)
                                 : reinterpret_cast<const void *>(k_coop_convert_segs<KPT, false>);
    const hipError_t e = coop_allow_lds(kernel, CP_SEGS_LDS_BYTES(KPT), asked[sym_nib ? 1 : 0]);
    if (e != hipSuccess) return e;
    if (sym_nib)
        hipLaunchKernelGGL((k_coop_convert_segs<KPT, true>), dim3(grid), dim3(CP_BLOCK), CP_SEGS_LDS_BYTES(KPT), st, g, err, sym, n,
                           stride, U, seg_off, nseg, anchor, gamma, fmt, counts, slots, tmax, spin_limit, status);
    else
        hipLaunchKernelGGL((k_coop_convert_segs<KPT, false>), dim3(grid), dim3(CP_BLOCK), CP_SEGS_LDS_BYTES(KPT), st, g, err, sym, n,
                           stride, U, seg_off, nseg, anchor, gamma, fmt, counts, slots, tmax, spin_limit, status);
    return hipGetLastError();
}

// `tmax`: U * nseg zero words (nseg > 1 only).  seg_off == nullptr or nseg == 1: one anchor per user.
hipError_t co3_launch_coop_convert(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int kpt,
                                   int grid, const int64_t *seg_off, int nseg, int32_t *anchor, float gamma, co3_fmt fmt,
                                   uint32_t *counts, uint32_t *slots, uint32_t *tmax, uint32_t spin_limit, int32_t *status,
                                   int sym_nib, hipStream_t st)
{
    if (seg_off && nseg > 1) {
        if (!tmax || nseg + 1 > CO3_SEG_CACHE) return hipErrorInvalidValue;
        Co3LaunchTimer tm(CO3_K_COOP, st);
#define CO3_COOP_SEGS_CASE(KPT)                                                                                    \
    case KPT:                                                                                                      \
        return coop_launch_segs<KPT>(g, err, sym, n, U, stride, grid, seg_off, nseg, anchor, gamma, fmt, counts, slots,  \
                                     tmax, spin_limit, status, sym_nib, st)
        switch (kpt) {
            CO3_COOP_SEGS_CASE(1);
            CO3_COOP_SEGS_CASE(4);
            CO3_COOP_SEGS_CASE(12);
            CO3_COOP_SEGS_CASE(CP_KPT_MAX);
            CO3_COOP_SEGS_CASE(CP_KPT_REG_MAX);
        default: return hipErrorInvalidValue;
        }
#undef CO3_COOP_SEGS_CASE
        return hipGetLastError();
    }
    {
    Co3LaunchTimer tm(CO3_K_COOP, st);
#define CO3_COOP_CASE(KPT)                                                                                         \
    case KPT:                                                                                                      \
        coop_launch_kpt<KPT>(g, err, sym, n, U, stride, grid, anchor, gamma, fmt, counts, slots, spin_limit, status, sym_nib, \
                             st);                                                                                  \
        break
    switch (kpt) {
        CO3_COOP_CASE(1);
        CO3_COOP_CASE(2);
        CO3_COOP_CASE(4);
        CO3_COOP_CASE(8);
        CO3_COOP_CASE(12);
        CO3_COOP_CASE(16);
        CO3_COOP_CASE(CP_KPT_MAX);
        CO3_COOP_CASE(CP_KPT_REG_MAX);
    case CP_BIG_KPT_SMALL:
        if (coop_launch_big<CP_BIG_KL_SMALL>(g, err, sym, n, U, stride, grid, anchor, gamma, fmt, counts, slots, spin_limit,
                                              status, sym_nib, st) != hipSuccess)
            return hipGetLastError();
        break;
    case CP_BIG_KPT:
        if (coop_launch_big<CP_BIG_KL>(g, err, sym, n, U, stride, grid, anchor, gamma, fmt, counts, slots, spin_limit, status,
                                        sym_nib, st) != hipSuccess)
            return hipGetLastError();
        break;
    default: return hipErrorInvalidValue;
    }
#undef CO3_COOP_CASE
    }
    // (the ragged end of the vector -- what the last wavefront with elements holds when these are fewer than
    // its kpt runs -- is left to the kernel that finishes the users, co3_launch_user_finish)
    return hipGetLastError();
}
