// The user's steps of Algorithm 1 (error correction, fp conversion, memory update, symbol statistics,
// Huffman code, compression) in ONE resident grid that reads every input once and writes every output
// once.  Two dependencies stand against that: the exponent anchor of a user needs the largest magnitude
// of the whole vector before the first element can be converted, and the user's code needs the counts
// of all symbols before the first one can be coded.  Kernels of their own for each step re-read g for
// the anchor and spill the symbols to memory to read them back twice.  Here one workgroup of 512 lanes
// per compute unit owns the same contiguous 1/G of every user's vector and keeps, between the steps,
//   - its part of the user's gradient in registers (largest magnitude first, conversion later), refilled
//     with the next user's gradient register by register as the conversion goes on,
//   - its part of the user's symbols in LDS until the user's code is known,
// and the workgroups exchange what depends on the whole vector through a few words of global memory:
//   A  largest magnitude      one word per workgroup              -> anchor
//   B  symbol counts          atomics into partial tables, then an arrival word per workgroup
//      code                   built by one wavefront of one workgroup (a different one for every user),
//                             which publishes the table of codewords
//   C  coded size and the first 64 stream bits of every workgroup's part -> stream positions, and the
//                             bits that complete a workgroup's last word
// No exchange uses a fence (a release or acquire at device scope writes back or invalidates a whole L2):
// every exchanged word validates itself -- a bit that the zeroed workspace does not have -- and is written
// with one relaxed device-scope store (the counts: relaxed device-scope atomics whose returned values the
// workgroup waits for before it publishes its arrival word), and read with relaxed device-scope loads.
// Every wait is bounded: after `spin_limit` polls the workgroup raises CO3_ETIMEOUT and goes on with
// harmless values (results are then unspecified, but in bounds, and the grid drains).
//
// The steps of user p that follow its conversion (code, sizes, positions, packing) run one user behind,
// after the exchange for user p + 1's anchor, so that the exchanges they wait for were started long before.
#include "co3_dev.h"
#include "co3_huffman.h"
#include "kernels.h"

#define CP_BLOCK 512
#define CP_WAVES (CP_BLOCK / CO3_WAVE)
#define CP_VEC 4
#define CP_STEP (CO3_WAVE * CP_VEC)          // elements that one load of a wavefront covers: one KiB
#define CP_KPT_MAX CO3_COOP_KPT_MAX          // steps per lane: 16-byte pieces of g that a lane keeps in registers
#ifndef CP_AHEAD
#define CP_AHEAD 6                           // memory loads in flight per lane ahead of the conversion
#endif
#define CP_HIST_SLOTS 512                    // LDS counters per wavefront
#define CP_VALID 0x80000000u
#define CP_VALID64 (1ull << 63)
#define CP_TILE CO3_PACK_SYMS                // symbols that a wavefront packs at a time (16 per lane)
#define CP_STAGE_WORDS 128                   // staging window of a wavefront: 8192 bits

__device__ __forceinline__ uint32_t ld_relaxed_agent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_relaxed_agent(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed_agent(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed_agent(uint64_t *p, uint64_t v)
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

// What the kernel is given (one struct: the argument list of a launch stays short).
struct CoopArgs {
    const float *g;
    float *err;
    uint8_t *sym;              // optional
    int64_t n, stride;
    int U;
    int32_t *anchor;           // [U] out
    float gamma;
    co3_fmt fmt;
    uint32_t *counts;          // [U][K] out
    char *codes;               // [U] code blobs out
    uint64_t *words;           // [U][cap_words] out
    int64_t cap_words;
    int chunk_syms;
    uint64_t *chunk_bitoff;    // [U][nchunks + 1] out
    int64_t nchunks;
    uint64_t *total_bits;      // [U] out
    // exchange words, zero when the kernel starts
    uint32_t *slots_a;         // [U][G]      valid | magnitude bits
    uint32_t *slots_b;         // [U][G]      valid
    uint32_t *cnt_rep;         // [CO3_COOP_COUNT_REPS][U][K] partial counts
    uint64_t *code_pub;        // [U][256]    valid | (codeword << 6 | length)
    uint64_t *slots_c;         // [U][G][2]   valid | size << 32 | head bits 63..32 ;  valid | head bits 31..0
    uint32_t spin_limit;
    int32_t *status;
};

// LDS of a workgroup
template <int KPT>
struct CoopLds {
    uint32_t hist[CP_WAVES][CP_HIST_SLOTS];        // counters of the user being converted, replicated per symbol
    uint32_t wavecnt[2][CP_WAVES][256];            // symbol counts of every wavefront's part: this user / the one before
    uint64_t enc[256];                             // (codeword << 6 | length) of the user being packed
    unsigned long long stage[CP_WAVES][CP_STAGE_WORDS];
    Co3BuildLds build;
    unsigned long long head;                       // first 64 stream bits of the workgroup's part
    uint64_t wg_base, head_next;                   // stream position of the workgroup's part; head of the next workgroup's
    uint32_t red[CP_WAVES + 1];
    uint32_t wavebits[CP_WAVES];
    uint32_t maxlen;
    __attribute__((aligned(16))) uint8_t sym[2][KPT * CP_WAVES * CP_STEP + 64];   // the workgroup's symbols, this user / the one before
};

// Polls (bounded) until `ready()` holds for every lane of the calling wavefront; returns whether it did.
template <class Ready>
__device__ __forceinline__ bool coop_wait(Ready ready, uint32_t spin_limit)
{
    uint32_t polls = 0;
    bool done = false;
    while (!done && polls < spin_limit) {
        done = __all(ready());
        ++polls;
        if (!done) __builtin_amdgcn_s_sleep(1);
    }
    return done;
}

// ---- exchange A: largest magnitude ------------------------------------------------------------------
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

// Waits until every workgroup's slot of the row is valid; returns the largest magnitude pattern over all
// of them to every lane of the workgroup (0 after a wait that ran out).
__device__ __forceinline__ uint32_t coop_collect_max(const uint32_t *row, int G, uint32_t spin_limit, uint32_t *red,
                                                     int32_t *status)
{
    if (threadIdx.x < CO3_WAVE) {
        const int lane = threadIdx.x;
        uint32_t m = 0;
        const bool done = coop_wait([&]() {
            bool all = true;
            m = 0;
            for (int j = lane; j < G; j += CO3_WAVE) {
                const uint32_t v = ld_relaxed_agent(row + j);
                all &= (v & CP_VALID) != 0u;
                const uint32_t a = v & ~CP_VALID;
                m = m > a ? m : a;
            }
            return all;
        }, spin_limit);
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

// ---- conversion ------------------------------------------------------------------------------------
// One user's conversion by one wavefront: KPT runs of 256 elements, the gradient from registers, the memory
// streamed CP_AHEAD runs ahead; as soon as a run is converted its registers take the next user's gradient.
// FULL: all KPT runs lie below n (straight-line code: the compiler can count the memory operations in
// flight exactly); else every access is guarded.  `left` = n - (first element of the wavefront's run 0).
struct CoopWave {
    float *eu;                 // the user's memory at the wavefront's run 0
    uint8_t *su;               // its symbols in global memory there, or NULL
    uint8_t *sl;               // its symbols in LDS there
    const float *gnext;        // the next user's gradient there (read when `more`)
    bool more;
    int64_t left;
    uint32_t lane4;
    int A, e_min, E, M, codemax;
    float gamma;
    uint32_t *myhist;
    int copies, mycopy;
};

template <int KPT, bool FULL>
__device__ __forceinline__ void coop_convert_user(const CoopWave &w, float4 (&gr)[KPT], float4 (&ev)[CP_AHEAD])
{
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        const int64_t rem = w.left - (int64_t)k * CP_STEP;                 // uniform: elements of this run below n
        float *ek = w.eu + k * CP_STEP;
        const float4 gv = gr[k], e4 = ev[k % CP_AHEAD];
        if (k + CP_AHEAD < KPT)
            ev[k % CP_AHEAD] = FULL ? ld_stream_f4(ek + CP_AHEAD * CP_STEP + w.lane4)
                                    : ld4_run(ek + CP_AHEAD * CP_STEP, rem - CP_AHEAD * CP_STEP, w.lane4);
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
        const uint32_t q4 = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        // the workgroup's copy of the symbols (entries past n are never read back)
        *reinterpret_cast<uint32_t *>(w.sl + k * CP_STEP + w.lane4) = q4;
        if (FULL || rem >= CP_STEP) {                             // uniform: the whole run exists
            st_stream_f4(ek + w.lane4, make_float4(en[0], en[1], en[2], en[3]));
            if (w.su) *reinterpret_cast<uint32_t *>(w.su + k * CP_STEP + w.lane4) = q4;
#pragma unroll
            for (int c = 0; c < CP_VEC; ++c) atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
        } else {
#pragma unroll
            for (int c = 0; c < CP_VEC; ++c)
                if ((int64_t)(w.lane4 + c) < rem) {
                    ek[w.lane4 + c] = en[c];
                    if (w.su) w.su[k * CP_STEP + w.lane4 + c] = (uint8_t)q[c];
                    atomicAdd(&w.myhist[q[c] * w.copies + w.mycopy], 1u);
                }
        }
        // the registers are free: the next user's gradient moves in
        if (w.more) gr[k] = FULL ? ld_stream_f4(w.gnext + k * CP_STEP + w.lane4) : ld4_run(w.gnext + k * CP_STEP, rem, w.lane4);
    }
}

// ---- packing -----------------------------------------------------------------------------------------
// ORs `nb` bits (right-aligned in `acc`, 1 <= nb <= 64) into the staging window at stream position `pos`
// (bits, relative to the first word of the tile); only words inside the window are touched.
__device__ __forceinline__ void coop_stage_bits(unsigned long long *stage, int64_t win_w0, uint64_t acc, int nb, uint64_t pos)
{
    const uint64_t v = acc << (64 - nb);
    const int64_t w = (int64_t)(pos >> 6) - win_w0;
    const int o = (int)(pos & 63);
    if (w >= 0 && w < CP_STAGE_WORDS) atomicOr(&stage[w], (unsigned long long)(v >> o));
    if (o + nb > 64 && w + 1 >= 0 && w + 1 < CP_STAGE_WORDS) atomicOr(&stage[w + 1], (unsigned long long)(v << (64 - o)));
}

// One wavefront packs a tile: `nsym` <= 1024 consecutive symbols at `syms` (LDS, 16 per lane) whose first bit
// has stream position B0, with the table enc (LDS).  It writes every word of the user's stream wu whose
// first bit lies in the tile; the last such word is completed with the codewords of the `ahead` (< 64)
// symbols that follow the tile in LDS and, where fewer than 63 symbols follow in the workgroup's part, with
// `tail_head` (the next workgroup's leading stream bits; zero after the last symbol of the vector).
// elem0: index of the tile's first symbol in the user's vector (chunk index).  Returns the tile's coded size.
__device__ __forceinline__ uint32_t coop_pack_tile(const uint8_t *syms, int nsym, int ahead, uint64_t tail_head,
                                                   const uint64_t *enc, uint32_t maxlen, uint64_t B0, uint64_t *wu,
                                                   int64_t cap_words, unsigned long long *stage, int lane, int64_t elem0,
                                                   int chunk_syms, uint64_t *chunk_bitoff_u)
{
    constexpr int LSYM = CP_TILE / CO3_WAVE;      // 16 symbols per lane
    int nvalid = nsym - lane * LSYM;
    nvalid = nvalid < 0 ? 0 : nvalid > LSYM ? LSYM : nvalid;
    uint32_t s[4] = {0u, 0u, 0u, 0u};
    if (nvalid > 0) {
        const uint4 a = *reinterpret_cast<const uint4 *>(syms + lane * LSYM);
        s[0] = a.x; s[1] = a.y; s[2] = a.z; s[3] = a.w;
    }
    const bool has_next = lane < CO3_WAVE - 1 && lane < ahead;
    const uint32_t next_sym = has_next ? syms[nsym + lane] : 0u;

    // codewords of the lane's symbols, four at a time joined into one run where they fit 64 bits
    uint64_t run[LSYM / 4];
    uint32_t runbits[LSYM / 4];
    uint32_t mybits = 0;
    bool wide = false;
    if (maxlen <= 16u && nsym == CP_TILE) {        // two codewords fit 32 bits: pairs joined with 32-bit operations
        const uint32_t *enc32 = reinterpret_cast<const uint32_t *>(enc);
#pragma unroll
        for (int g = 0; g < LSYM / 4; ++g) {
            const uint32_t e0 = enc32[2 * (s[g] & 0xffu)], e1 = enc32[2 * ((s[g] >> 8) & 0xffu)];
            const uint32_t e2 = enc32[2 * ((s[g] >> 16) & 0xffu)], e3 = enc32[2 * (s[g] >> 24)];
            const uint32_t l1 = e1 & 63u, l3 = e3 & 63u;
            const uint32_t p01 = ((e0 >> 6) << l1) | (e1 >> 6);
            const uint32_t p23 = ((e2 >> 6) << l3) | (e3 >> 6);
            const uint32_t n23 = (e2 & 63u) + l3;
            const uint32_t nb = (e0 & 63u) + l1 + n23;
            run[g] = ((uint64_t)p01 << n23) | (uint64_t)p23;
            runbits[g] = nb;
            mybits += nb;
        }
    } else {
#pragma unroll
        for (int g = 0; g < LSYM / 4; ++g) {
            uint64_t acc = 0;
            uint32_t nb = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t e = 4 * g + k < nvalid ? enc[(s[g] >> (8 * k)) & 0xffu] : 0ull;
                const uint32_t l = (uint32_t)(e & 63u);
                acc = (acc << l) | (e >> 6);
                nb += l;
            }
            wide |= nb > 64u;
            run[g] = acc;
            runbits[g] = nb;
            mybits += nb;
        }
    }
    const uint32_t incl = wave_scan_incl_u32(mybits, lane);
    const uint32_t excl = incl - mybits;
    const uint32_t tilebits = (uint32_t)__builtin_amdgcn_readlane((int)incl, CO3_WAVE - 1);
    const uint64_t B1 = B0 + tilebits;

    // chunk index: stream position of every chunk that starts at this lane's first symbol
    const int64_t i = elem0 + (int64_t)lane * LSYM;
    if (nvalid > 0 && (i & (int64_t)(chunk_syms - 1)) == 0) chunk_bitoff_u[i / chunk_syms] = B0 + excl;
    // beyond the capacity nothing is written (reported where the stream length is known); uniform
    if ((B1 + 63) / 64 > (uint64_t)cap_words || tilebits == 0) return tilebits;

    const int64_t gw0 = (int64_t)(B0 >> 6);          // first and last stream word the tile touches
    const int64_t gwl = (int64_t)((B1 - 1) >> 6);
    const int64_t first_owned = (B0 & 63) ? gw0 + 1 : gw0;   // words whose first bit lies in the tile
    const uint64_t rel0 = (B0 & 63) + excl;          // position of this lane's bits, relative to word gw0

    // what completes the last word: the codewords of the symbols after the tile, then the next workgroup's bits
    auto complete_last = [&](int64_t last_rel) {
        const uint32_t used = (uint32_t)(B1 & 63);
        const uint64_t e = has_next ? enc[next_sym] : 0ull;
        const uint32_t l = (uint32_t)(e & 63u);
        const uint32_t io = wave_scan_incl_u32(l, lane);
        const uint32_t o = io - l;
        if (l && used + o < 64u) atomicOr(&stage[last_rel], (unsigned long long)(((e >> 6) << (64 - l)) >> (used + o)));
        const uint32_t after = used + (uint32_t)__builtin_amdgcn_readlane((int)io, CO3_WAVE - 1);   // bits in the word so far
        if (lane == 0 && ahead < CO3_WAVE - 1 && after < 64u) atomicOr(&stage[last_rel], (unsigned long long)(tail_head >> after));
    };

    if ((B0 & 63) + tilebits <= CP_STAGE_WORDS * 64u && !__any(wide)) {
        // usual case: the tile fits one staging window and every run fits 64 bits
#pragma unroll
        for (int j = 0; j < CP_STAGE_WORDS / CO3_WAVE; ++j) stage[lane + j * CO3_WAVE] = 0ull;
        co3_wave_lds_sync();
        uint32_t pos = (uint32_t)rel0;
#pragma unroll
        for (int g = 0; g < LSYM / 4; ++g) {
            const uint32_t nb = runbits[g];
            if (nb) {
                const uint64_t v = run[g] << (64u - nb);
                const uint32_t w = pos >> 6, o = pos & 63u;
                atomicOr(&stage[w], (unsigned long long)(v >> o));
                if (o + nb > 64u) atomicOr(&stage[w + 1], (unsigned long long)(v << (64u - o)));
            }
            pos += nb;
        }
        const uint32_t last_rel = (uint32_t)(gwl - gw0);
        if (B1 & 63) complete_last(last_rel);
        co3_wave_lds_sync();
        const uint32_t first_rel = (uint32_t)(first_owned - gw0);
#pragma unroll
        for (int j = 0; j < CP_STAGE_WORDS / CO3_WAVE; ++j) {
            const uint32_t r = lane + j * CO3_WAVE;
            if (r >= first_rel && r <= last_rel) wu[gw0 + r] = stage[r];
        }
        co3_wave_lds_sync();                         // the window is reused by the next tile
        return tilebits;
    }

    for (int64_t win_w0 = 0; gw0 + win_w0 <= gwl; win_w0 += CP_STAGE_WORDS) {
#pragma unroll
        for (int j = 0; j < CP_STAGE_WORDS / CO3_WAVE; ++j) stage[lane + j * CO3_WAVE] = 0ull;
        co3_wave_lds_sync();
        if (!wide) {
            uint64_t pos = rel0;
#pragma unroll
            for (int g = 0; g < LSYM / 4; ++g) {
                if (runbits[g]) coop_stage_bits(stage, win_w0, run[g], (int)runbits[g], pos);
                pos += runbits[g];
            }
        } else {
            // runs of at most 64 bits, symbol by symbol
            uint64_t acc = 0, pos = rel0;
            int accbits = 0;
            for (int c = 0; c < nvalid; ++c) {
                const uint64_t e = enc[(s[c >> 2] >> (8 * (c & 3))) & 0xffu];
                const int l = (int)(e & 63u);
                if (l) {
                    if (accbits + l > 64) {
                        coop_stage_bits(stage, win_w0, acc, accbits, pos);
                        pos += accbits;
                        acc = 0;
                        accbits = 0;
                    }
                    acc = (acc << l) | (e >> 6);
                    accbits += l;
                }
            }
            if (accbits) coop_stage_bits(stage, win_w0, acc, accbits, pos);
        }
        const int64_t last_rel = gwl - gw0 - win_w0;
        if ((B1 & 63) && last_rel >= 0 && last_rel < CP_STAGE_WORDS) complete_last(last_rel);
        co3_wave_lds_sync();
#pragma unroll
        for (int j = 0; j < CP_STAGE_WORDS / CO3_WAVE; ++j) {
            const int64_t gw = gw0 + win_w0 + lane + j * CO3_WAVE;
            if (gw >= first_owned && gw <= gwl) wu[gw] = stage[lane + j * CO3_WAVE];
        }
        co3_wave_lds_sync();
    }
    return tilebits;
}

// ---- the steps of user p after its conversion ----------------------------------------------------------
// Called by the whole workgroup (it contains workgroup barriers); pb = p & 1 selects the LDS copies of p.
template <int KPT>
__device__ __forceinline__ void coop_finish_user(const CoopArgs &a, CoopLds<KPT> &lds, int p, int G, int K, int wave, int lane)
{
    const int pb = p & 1;
    const int64_t wg_first = (int64_t)blockIdx.x * KPT * CP_WAVES * CP_STEP;            // the workgroup's first element
    const int64_t wg_left = a.n - wg_first;
    const int wg_nsym = wg_left <= 0 ? 0 : wg_left > KPT * CP_WAVES * CP_STEP ? KPT * CP_WAVES * CP_STEP : (int)wg_left;
    uint64_t *pub = a.code_pub + (int64_t)p * 256;

    // 1. the code: one wavefront of workgroup p mod G adds the partial tables up and builds it
    if ((int)blockIdx.x == p % G && wave == 1) {
        const uint32_t *row = a.slots_b + (int64_t)p * G;
        const bool done = coop_wait([&]() {
            bool all = true;
            for (int j = lane; j < G; j += CO3_WAVE) all &= (ld_relaxed_agent(row + j) & CP_VALID) != 0u;
            return all;
        }, a.spin_limit);
        if (!done && lane == 0) co3_raise(a.status, CO3_ETIMEOUT);
        uint32_t wt[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = lane + j * CO3_WAVE;
            if (s < K) {
                for (int r0 = 0; r0 < CO3_COOP_COUNT_REPS; r0 += 8) {      // eight loads in flight
                    uint32_t part[8];
#pragma unroll
                    for (int r = 0; r < 8; ++r) part[r] = ld_relaxed_agent(a.cnt_rep + ((int64_t)(r0 + r) * a.U + p) * K + s);
#pragma unroll
                    for (int r = 0; r < 8; ++r) wt[j] += part[r];
                }
                a.counts[(int64_t)p * K + s] = wt[j];
            }
        }
        co3_build_code_group<CO3_WAVE>(lds.build, lane, wt, K, reinterpret_cast<Co3Code *>(a.codes + (size_t)p * CO3_CODE_BYTES),
                                       pub, a.status, Co3WaveSync());
    }
    // 2. every workgroup takes the published table
    if (wave == 2) {
        uint64_t e[4] = {0ull, 0ull, 0ull, 0ull};
        const bool done = coop_wait([&]() {
            bool all = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int s = lane + j * CO3_WAVE;
                if (s < K) {
                    e[j] = ld_relaxed_agent(pub + s);
                    all &= (e[j] & CP_VALID64) != 0ull;
                }
            }
            return all;
        }, a.spin_limit);
        if (!done && lane == 0) co3_raise(a.status, CO3_ETIMEOUT);
        uint32_t ml = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t v = done ? e[j] & ~CP_VALID64 : 0ull;      // after a wait that ran out: no codewords, no bits
            lds.enc[lane + j * CO3_WAVE] = v;
            const uint32_t l = (uint32_t)(v & 63u);
            ml = ml > l ? ml : l;
        }
        ml = wave_max_u32(ml);
        if (lane == 0) {
            lds.maxlen = ml;
            lds.head = 0ull;
        }
    }
    __syncthreads();

    // 3. coded size of every wavefront's part from its symbol counts; first 64 stream bits of the workgroup's part
    {
        uint32_t bits = 0;
        for (int k = lane; k < K; k += CO3_WAVE) bits += lds.wavecnt[pb][wave][k] * (uint32_t)(lds.enc[k] & 63u);
        bits = wave_sum_u32(bits);
        if (lane == 0) lds.wavebits[wave] = bits;
    }
    if (wave == 3) {
        const uint64_t e = lane < wg_nsym ? lds.enc[lds.sym[pb][lane]] : 0ull;
        const uint32_t l = (uint32_t)(e & 63u);
        const uint32_t o = wave_scan_incl_u32(l, lane) - l;
        if (l && o < 64u) atomicOr(&lds.head, (unsigned long long)(((e >> 6) << (64 - l)) >> o));
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
#pragma unroll
        for (int v = 0; v < CP_WAVES; ++v) total += lds.wavebits[v];
        const uint64_t head = lds.head;
        uint64_t *c = a.slots_c + ((int64_t)p * G + blockIdx.x) * 2;
        st_relaxed_agent(c + 0, CP_VALID64 | ((uint64_t)total << 32) | (head >> 32));
        st_relaxed_agent(c + 1, CP_VALID64 | (head & 0xffffffffull));
    }
    // 4. stream position of the workgroup's part; the next workgroup's leading bits
    if (wave == 3) {
        const uint64_t *row = a.slots_c + (int64_t)p * G * 2;
        uint64_t before = 0, all_bits = 0, hn0 = 0, hn1 = 0;
        const bool done = coop_wait([&]() {
            bool all = true;
            before = 0;
            all_bits = 0;
            for (int j = lane; j < G; j += CO3_WAVE) {
                const uint64_t v = ld_relaxed_agent(row + 2 * j);
                all &= (v & CP_VALID64) != 0ull;
                const uint64_t sz = (v >> 32) & 0x7fffffffull;
                all_bits += sz;
                before += j < (int)blockIdx.x ? sz : 0ull;
            }
            if (lane == 0 && (int)blockIdx.x + 1 < G) {
                hn0 = ld_relaxed_agent(row + 2 * (blockIdx.x + 1));
                hn1 = ld_relaxed_agent(row + 2 * (blockIdx.x + 1) + 1);
                all &= (hn0 & CP_VALID64) != 0ull && (hn1 & CP_VALID64) != 0ull;
            }
            return all;
        }, a.spin_limit);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            before += (uint64_t)__shfl_xor((long long)before, o, CO3_WAVE);
            all_bits += (uint64_t)__shfl_xor((long long)all_bits, o, CO3_WAVE);
        }
        if (lane == 0) {
            if (!done) {
                co3_raise(a.status, CO3_ETIMEOUT);
                before = ~0ull >> 1;           // beyond every capacity: nothing is written
            }
            lds.wg_base = before;
            lds.head_next = (int)blockIdx.x + 1 < G ? ((hn0 & 0xffffffffull) << 32) | (hn1 & 0xffffffffull) : 0ull;
            if (blockIdx.x == 0 && done) {
                a.total_bits[p] = all_bits;
                a.chunk_bitoff[(int64_t)p * (a.nchunks + 1) + a.nchunks] = all_bits;
                if ((all_bits + 63) / 64 > (uint64_t)a.cap_words) co3_raise(a.status, CO3_ECAP);
            }
        }
    }
    __syncthreads();

    // 5. every wavefront packs its part, tile by tile
    {
        const int part = KPT * CP_STEP;                       // symbols of a wavefront's part
        const int w0 = wave * part;                           // its first symbol within the workgroup's
        int nsym_wave = wg_nsym - w0;
        nsym_wave = nsym_wave < 0 ? 0 : nsym_wave > part ? part : nsym_wave;
        uint64_t B0 = lds.wg_base;
        for (int v = 0; v < wave; ++v) B0 += lds.wavebits[v];
        const uint32_t maxlen = lds.maxlen;
        const uint64_t head_next = lds.head_next;
        uint64_t *wu = a.words + (int64_t)p * a.cap_words;
        uint64_t *cbu = a.chunk_bitoff + (int64_t)p * (a.nchunks + 1);
        for (int t0 = 0; t0 < nsym_wave; t0 += CP_TILE) {
            const int nsym = nsym_wave - t0 < CP_TILE ? nsym_wave - t0 : CP_TILE;
            int ahead = wg_nsym - (w0 + t0 + nsym);           // symbols of the workgroup after the tile
            ahead = ahead > CO3_WAVE - 1 ? CO3_WAVE - 1 : ahead;
            B0 += coop_pack_tile(lds.sym[pb] + w0 + t0, nsym, ahead, head_next, lds.enc, maxlen, B0, wu, a.cap_words,
                                 lds.stage[wave], lane, wg_first + w0 + t0, a.chunk_syms, cbu);
        }
    }
    __syncthreads();          // enc, wavebits and the symbols of p are free
}

// grid: G workgroups (at most one per compute unit, all resident); workgroup w owns elements
// [w * KPT * 2048, (w + 1) * KPT * 2048) of every user, wavefront v of it the v-th eighth, lane l of the
// wavefront elements 4l .. 4l+3 of each of the wavefront's KPT runs of 256.
template <int KPT>
__global__ __launch_bounds__(CP_BLOCK) void k_coop_user(const CoopArgs a)
{
    const FmtC fc(a.fmt);
    const int F = fc.F, K = fc.K;
    const int G = gridDim.x, U = a.U;
    const int64_t n = a.n;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / CO3_WAVE);     // uniform: addresses of a run are scalar
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    CoopLds<KPT> &lds = *reinterpret_cast<CoopLds<KPT> *>(lds_raw);
    const int copies = CP_HIST_SLOTS / K > 32 ? 32 : CP_HIST_SLOTS / K;
    for (int j = threadIdx.x; j < CP_WAVES * CP_HIST_SLOTS; j += CP_BLOCK) (&lds.hist[0][0])[j] = 0u;

    // first element of the wavefront's run 0 (uniform); run k lies k * CP_STEP further
    const int64_t first = (((int64_t)blockIdx.x * CP_WAVES + wave) * KPT) * CP_STEP;
    const uint32_t lane4 = (uint32_t)lane * CP_VEC;
    const bool full = first + (int64_t)KPT * CP_STEP <= n;      // uniform: every run of the wavefront is whole

    // user 0's gradient: every load of the lane in flight at once
    float4 gr[KPT];
    if (full) {
#pragma unroll
        for (int k = 0; k < KPT; ++k) gr[k] = ld_stream_f4(a.g + first + k * CP_STEP + lane4);
    } else {
#pragma unroll
        for (int k = 0; k < KPT; ++k) gr[k] = ld4_run(a.g + first + k * CP_STEP, n - first - k * CP_STEP, lane4);
    }
    {
        uint32_t m = 0;
#pragma unroll
        for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
        coop_publish_max(m, a.slots_a, lds.red);
    }

    CoopWave w;
    w.left = n - first;
    w.lane4 = lane4;
    w.E = fc.E;
    w.M = fc.M;
    w.codemax = fc.codemax;
    w.gamma = a.gamma;
    w.myhist = lds.hist[wave];
    w.copies = copies;
    w.mycopy = lane & (copies - 1);
    for (int u = 0; u < U; ++u) {
        const int ub = u & 1;
        w.gnext = a.g + (int64_t)(u + 1) * a.stride + first;          // only read when u + 1 < U
        w.eu = a.err + (int64_t)u * a.stride + first;
        w.su = a.sym ? a.sym + (int64_t)u * a.stride + first : nullptr;
        w.sl = lds.sym[ub] + (wave * KPT) * CP_STEP;
        w.more = u + 1 < U;

        const uint32_t mm = coop_collect_max(a.slots_a + (int64_t)u * G, G, a.spin_limit, lds.red, a.status);
        int A = (int)(mm >> 23) - 127;
        A = A > 127 ? 127 : A;
        A = A < F - 126 ? F - 126 : A;
        if (blockIdx.x == 0 && threadIdx.x == 0) a.anchor[u] = A;
        w.A = A;
        w.e_min = A - F + 1;

        // the user before this one: its counts were published when its conversion ended
        if (u > 0) coop_finish_user<KPT>(a, lds, u - 1, G, K, wave, lane);

        float4 ev[CP_AHEAD];
        if (full) {
#pragma unroll
            for (int k = 0; k < CP_AHEAD; ++k)
                ev[k] = k < KPT ? ld_stream_f4(w.eu + k * CP_STEP + lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
#pragma unroll
            for (int k = 0; k < CP_AHEAD; ++k)
                ev[k] = k < KPT ? ld4_run(w.eu + k * CP_STEP, w.left - k * CP_STEP, lane4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }

        if (full) coop_convert_user<KPT, true>(w, gr, ev);
        else coop_convert_user<KPT, false>(w, gr, ev);

        if (w.more) {
            uint32_t m = 0;
#pragma unroll
            for (int k = 0; k < KPT; ++k) m = absbits4(gr[k], m);
            coop_publish_max(m, a.slots_a + (int64_t)(u + 1) * G, lds.red);
        }
        // The workgroup's counts of this user.  Entry j of a wavefront's counters = symbol * copies + replica:
        // a lane takes entry j of every wavefront, the lanes of one symbol (consecutive) are summed by exchange,
        // the sums stay in LDS (coded size of the wavefront's part, later) and go to one of several partial
        // tables in global memory (every workgroup adding to the same K words at the same moment serialises
        // chip-wide, and the loads behind the atomics wait).
        __syncthreads();
        for (int j = threadIdx.x; j < K * copies; j += CP_BLOCK) {       // whole wavefronts take part or not
            uint32_t tot = 0;
#pragma unroll
            for (int wv = 0; wv < CP_WAVES; ++wv) {
                uint32_t c = lds.hist[wv][j];
                lds.hist[wv][j] = 0u;
                for (int o = copies >> 1; o >= 1; o >>= 1) c += (uint32_t)__shfl_xor((int)c, o, CO3_WAVE);
                if ((j & (copies - 1)) == 0) lds.wavecnt[ub][wv][j / copies] = c;
                tot += c;
            }
            if ((j & (copies - 1)) == 0 && tot) {
                // the returned value is waited for: the arrival word below must not overtake the addition
                const uint32_t old = __hip_atomic_fetch_add(
                    a.cnt_rep + ((int64_t)(blockIdx.x % CO3_COOP_COUNT_REPS) * U + u) * K + j / copies, tot, __ATOMIC_RELAXED,
                    __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("" ::"v"(old));
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) st_relaxed_agent(a.slots_b + (int64_t)u * G + blockIdx.x, CP_VALID);
    }
    coop_finish_user<KPT>(a, lds, U - 1, G, K, wave, lane);
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

// 32-bit exchange words for U users on `grid` workgroups, padded to a whole number of 64-bit words
static size_t coop_words32(int U, int grid, int K)
{
    const size_t w = (size_t)U * grid * 2 + (size_t)CO3_COOP_COUNT_REPS * U * K;
    return (w + 1) & ~(size_t)1;
}

// bytes of exchange words (zeroed before every launch)
size_t co3_coop_exchange_bytes(int U, int grid, int K)
{
    return coop_words32(U, grid, K) * 4 + ((size_t)U * 256 + (size_t)U * grid * 2) * 8;
}

template <int KPT>
static hipError_t coop_launch_kpt(const CoopArgs &a, int grid, hipStream_t st)
{
    const size_t lds_bytes = sizeof(CoopLds<KPT>);
    // more than 64 KiB of LDS must be asked for once per kernel (setting it again is harmless)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_coop_user<KPT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_coop_user<KPT>), dim3(grid), dim3(CP_BLOCK), lds_bytes, st, a);
    return hipGetLastError();
}

hipError_t co3_launch_coop_user(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int kpt,
                                int grid, int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, void *codes,
                                uint64_t *words, int64_t cap_words, int chunk_syms, uint64_t *chunk_bitoff,
                                uint64_t *total_bits, void *exchange, uint32_t spin_limit, int32_t *status, hipStream_t st)
{
    const int K = 1 << (1 + fmt.exp_bits + fmt.mant_bits);
    // exchange words start at zero
    hipError_t e = co3_launch_fill(static_cast<int32_t *>(exchange), (int64_t)(co3_coop_exchange_bytes(U, grid, K) / 4), 0,
                                   nullptr, 0, st);
    if (e != hipSuccess) return e;
    CoopArgs a;
    a.g = g; a.err = err; a.sym = sym; a.n = n; a.stride = stride; a.U = U; a.anchor = anchor; a.gamma = gamma; a.fmt = fmt;
    a.counts = counts; a.codes = static_cast<char *>(codes); a.words = words; a.cap_words = cap_words; a.chunk_syms = chunk_syms;
    a.chunk_bitoff = chunk_bitoff; a.nchunks = (n + chunk_syms - 1) / chunk_syms; a.total_bits = total_bits;
    uint32_t *p32 = static_cast<uint32_t *>(exchange);
    a.slots_a = p32;
    a.slots_b = p32 + (size_t)U * grid;
    a.cnt_rep = p32 + (size_t)U * grid * 2;
    uint64_t *p64 = reinterpret_cast<uint64_t *>(p32 + coop_words32(U, grid, K));
    a.code_pub = p64;
    a.slots_c = p64 + (size_t)U * 256;
    a.spin_limit = spin_limit;
    a.status = status;
    Co3LaunchTimer tm(CO3_K_COOP, st);
    switch (kpt) {
    case 1: return coop_launch_kpt<1>(a, grid, st);
    case 2: return coop_launch_kpt<2>(a, grid, st);
    case 4: return coop_launch_kpt<4>(a, grid, st);
    case 8: return coop_launch_kpt<8>(a, grid, st);
    case 12: return coop_launch_kpt<12>(a, grid, st);
    case 16: return coop_launch_kpt<16>(a, grid, st);
    case CP_KPT_MAX: return coop_launch_kpt<CP_KPT_MAX>(a, grid, st);
    default: return hipErrorInvalidValue;
    }
}
