// User side of Algorithm 1 in one pass over g and the memory, for codes that are known before the
// iteration starts (tables designed from a model, Sec. III (ii), or kept from an earlier iteration):
// error correction, fp conversion and compression without the symbol array in between.
//
// The stream position of a codeword depends on all symbols before it, so the pass cannot write the
// stream itself.  Each wavefront converts a unit of 1024 consecutive elements (sixteen per lane), packs the
// unit's codewords from bit 0 of a private slot of the workspace and records the unit's length; a
// small kernel turns the lengths into offsets within groups of 64 units, the packer's scan kernel into
// stream offsets of the groups, and a last kernel moves every slot to its place in the stream (a funnel
// shift of whole words, the last word of a unit completed with the leading bits of the next unit, so
// that every word of the stream is written once, by one lane, with plain stores).
#include "co3_dev.h"
#include "kernels.h"

#define FU_BLOCK 256
#define FU_WAVES (FU_BLOCK / CO3_WAVE)
#define FU_VEC 4
#define FU_HIST_SLOTS 512                      // LDS counters per wavefront (optional symbol counts)
#define FU_RUN (CO3_WAVE * FU_VEC)              // consecutive elements that one load of a wavefront covers
#define FU_SUB (CO3_FUSED_UNIT / FU_RUN)        // runs per unit
#define FU_TILE (FU_WAVES * CO3_FUSED_UNIT)     // elements of one block step: four units, one per wavefront
static_assert(CO3_FUSED_UNIT % (2 * FU_RUN) == 0, "unit geometry: an even number of runs");
static_assert(FU_RUN * CO3_MAX_CODE_LEN < 65536, "the bits of a run fit 16 bits");
static_assert(CO3_FUSED_SLOT_WORDS * 64 >= CO3_FUSED_UNIT * CO3_MAX_CODE_LEN, "a slot holds any unit");

__device__ __forceinline__ const Co3Code *fcode_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// ORs `nb` bits (right-aligned in `acc`, 1 <= nb <= 64) into the unit's staging window at bit `pos`
__device__ __forceinline__ void fused_stage(unsigned long long *stage, uint64_t acc, uint32_t nb, uint32_t pos)
{
    const uint64_t v = acc << (64u - nb);
    const uint32_t w = pos >> 6, o = pos & 63u;
    atomicOr(&stage[w], (unsigned long long)(v >> o));
    if (o + nb > 64u) atomicOr(&stage[w + 1], (unsigned long long)(v << (64u - o)));
}

// One unit's elements: error correction, conversion, new memory, codeword lookup.  WHOLE: all 1024
// elements exist (vector loads and stores), else every access is guarded.  PLAIN (with WHOLE): they lie
// in one tensor and under one code (one anchor, one multiplier, the table in LDS, no branches between the
// elements, so that the table reads of a lane overlap); else anchor, multiplier and code are looked up
// per element.
// SCALED: the bias in its multiplier form (Sec. III (i), Sec. IV-B), as in the two-pass conversion: the
// corrected gradient times c is rounded onto the grid, the level divided by c.  LAYERS: one code per
// group of tensors (Sec. III (ii)), codes[group], the wavefront's LDS table holding the code of the
// unit's first element.  Returns whether a symbol without a codeword was met.
struct FusedUnit {
    const float *gu;
    float *eu;
    int64_t n, u0;
    int lane;
    const int64_t *seg_off;
    int nseg;
    const int32_t *anchor_u;
    const float *scale_u;
    int A_unit;
    float c_unit;
    float gamma;
    int E, M, F, K, codemax;
    const uint64_t *enc_s;
    const void *codes;
    const int64_t *code_seg_off;
    int ncodes;
    bool one_code;
    uint32_t *hist;      // the wavefront's LDS counters (HIST), slot of symbol q: q * copies + mycopy
    int copies, mycopy;
    uint32_t *counts;    // HIST with LAYERS: the pooled counters [ncodes][K] in global memory
};

template <bool LAYERS>
__device__ __forceinline__ uint64_t fused_entry(const FusedUnit &a, uint32_t q, int64_t idx)
{
    if (!LAYERS || a.one_code) return a.enc_s[q];
    return (int)q < a.K ? fcode_of(a.codes, co3_find_seg(a.code_seg_off, a.ncodes, idx))->enc[q] : 0ull;
}
// the same with the code groups of the first and the last of the lane's four consecutive elements known
template <bool LAYERS>
__device__ __forceinline__ uint64_t fused_entry4(const FusedUnit &a, uint32_t q, int64_t idx, int cg_first, int cg_last)
{
    if (!LAYERS || a.one_code) return a.enc_s[q];
    const int cg = cg_first == cg_last ? cg_first : co3_find_seg(a.code_seg_off, a.ncodes, idx);
    return (int)q < a.K ? fcode_of(a.codes, cg)->enc[q] : 0ull;
}

template <bool WHOLE, bool PLAIN, bool LAYERS, bool SCALED, bool HIST>
__device__ __forceinline__ bool fused_convert_unit(const FusedUnit &a, uint64_t (&acc)[FU_SUB], uint32_t (&qpack)[FU_SUB],
                                                   uint32_t (&nb)[FU_SUB])
{
    float4 gv[FU_SUB], ev[FU_SUB];
#pragma unroll
    for (int r = 0; r < FU_SUB; ++r) {
        const int64_t i = a.u0 + r * FU_RUN + a.lane * FU_VEC;
        if (WHOLE) {
            gv[r] = ld_stream_f4(a.gu + i);
            ev[r] = ld_stream_f4(a.eu + i);
        } else {
            gv[r].x = i + 0 < a.n ? a.gu[i + 0] : 0.0f; ev[r].x = i + 0 < a.n ? a.eu[i + 0] : 0.0f;
            gv[r].y = i + 1 < a.n ? a.gu[i + 1] : 0.0f; ev[r].y = i + 1 < a.n ? a.eu[i + 1] : 0.0f;
            gv[r].z = i + 2 < a.n ? a.gu[i + 2] : 0.0f; ev[r].z = i + 2 < a.n ? a.eu[i + 2] : 0.0f;
            gv[r].w = i + 3 < a.n ? a.gu[i + 3] : 0.0f; ev[r].w = i + 3 < a.n ? a.eu[i + 3] : 0.0f;
        }
    }
    bool nocode = false;
#pragma unroll
    for (int r = 0; r < FU_SUB; ++r) {
        const int64_t i = a.u0 + r * FU_RUN + a.lane * FU_VEC;
        const float ga[FU_VEC] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float ea[FU_VEC] = {ev[r].x, ev[r].y, ev[r].z, ev[r].w};
        float en[FU_VEC];
        acc[r] = 0;
        qpack[r] = 0;
        nb[r] = 0;
        // tensors and code groups of the lane's first and last element of the run: mostly the same
        int sg_first = 0, sg_last = 0, cg_first = 0, cg_last = 0;
        if (!PLAIN) {
            const int64_t j0 = i < a.n ? i : a.n - 1, j3 = i + FU_VEC - 1 < a.n ? i + FU_VEC - 1 : a.n - 1;
            sg_first = co3_find_seg(a.seg_off, a.nseg, j0);
            sg_last = co3_find_seg(a.seg_off, a.nseg, j3);
            if (LAYERS && !a.one_code) {
                cg_first = co3_find_seg(a.code_seg_off, a.ncodes, j0);
                cg_last = co3_find_seg(a.code_seg_off, a.ncodes, j3);
            }
        }
#pragma unroll
        for (int k = 0; k < FU_VEC; ++k) {
            const bool valid = WHOLE || i + k < a.n;
            const int64_t idx = valid ? i + k : a.n - 1;
            const int sg = PLAIN ? 0 : sg_first == sg_last ? sg_first : co3_find_seg(a.seg_off, a.nseg, idx);
            const int A = PLAIN ? a.A_unit : a.anchor_u[sg];
            const float c = !SCALED ? 1.0f : PLAIN ? a.c_unit : a.scale_u[sg];
            const float x = ga[k] + a.gamma * ea[k];     // no contraction (build flag): one rounding per operation
            uint32_t q;
            float v;
            co3_quantize(SCALED ? c * x : x, A - a.F + 1, A, a.E, a.M, a.codemax, q, v);
            if (SCALED) v = v / c;
            en[k] = x - v;
            if (HIST && valid) {
                if (!LAYERS || a.one_code) {
                    atomicAdd(&a.hist[q * a.copies + a.mycopy], 1u);
                } else {                 // a unit that straddles code groups: straight to the group's counters
                    const int cg = cg_first == cg_last ? cg_first : co3_find_seg(a.code_seg_off, a.ncodes, idx);
                    atomicAdd(&a.counts[(int64_t)cg * a.K + q], 1u);
                }
            }
            const uint64_t e = !valid ? 0ull : PLAIN ? a.enc_s[q] : fused_entry4<LAYERS>(a, q, idx, cg_first, cg_last);
            const uint32_t l = (uint32_t)(e & 63u);
            nocode |= valid && l == 0u;
            acc[r] = (acc[r] << l) | (e >> 6);
            qpack[r] |= q << (8 * k);
            nb[r] += l;
        }
        if (WHOLE) {
            st_stream_f4(a.eu + i, make_float4(en[0], en[1], en[2], en[3]));
        } else {
#pragma unroll
            for (int k = 0; k < FU_VEC; ++k)
                if (i + k < a.n) a.eu[i + k] = en[k];
        }
    }
    return nocode;
}

// Adds a wavefront's LDS counters (all replicas of every symbol) to K global counters and clears them.
__device__ __forceinline__ void flush_wave_counts(uint32_t *hist, int copies, int K, int lane, uint32_t *dst)
{
    for (int k = lane; k < K; k += CO3_WAVE) {
        uint32_t c = 0;
        for (int r = 0; r < copies; ++r) {
            c += hist[k * copies + r];
            hist[k * copies + r] = 0u;
        }
        if (c) atomicAdd(&dst[k], c);
    }
    co3_wave_lds_sync();
}

// ---- pass 1: conversion with error correction, codeword lookup, unit-local packing -----------
// A unit is FU_SUB runs of 256 elements; lane l holds elements 4l..4l+3 of every run, so each load is
// one contiguous KiB per wavefront.  The bit position of a lane's codewords inside the unit comes from
// one scan over the lanes for all runs at once: the lane totals of two runs share a 32-bit word (a run
// has at most 256 * 57 < 2^16 bits).
template <bool LAYERS, bool SCALED, bool HIST>
__global__ __launch_bounds__(FU_BLOCK) void k_convert_stage(const float *__restrict__ g, float *__restrict__ err,
                                                             int64_t n, int64_t stride,
                                                             const int64_t *__restrict__ seg_off_g, int nseg,
                                                             const int32_t *__restrict__ anchor,
                                                             const float *__restrict__ scale, float gamma, co3_fmt fmt,
                                                             const void *__restrict__ codes,
                                                             const int64_t *__restrict__ code_seg_off_g, int ncodes,
                                                             uint32_t *__restrict__ counts,
                                                             uint64_t *__restrict__ slots, uint32_t *__restrict__ unit_bits,
                                                             uint32_t *__restrict__ chunk_local, int chunk_syms,
                                                             int64_t nchunks, int64_t nunits, int64_t per_block,
                                                             int32_t *status)
{
    const FmtC fc(fmt);
    const int E = fc.E, M = fc.M, F = fc.F, K = fc.K, codemax = fc.codemax;
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    __shared__ int64_t code_seg_cache[LAYERS ? CO3_SEG_CACHE : 1];
    __shared__ uint64_t enc_all[LAYERS ? FU_WAVES * 256 : 256];
    __shared__ unsigned long long stage_all[FU_WAVES][CO3_FUSED_SLOT_WORDS + 1];
    // HIST: per-wavefront counters, `copies` interleaved replicas per symbol so that lanes that meet one
    // popular symbol spread over banks (as in the two-pass conversion)
    __shared__ uint32_t hist_all[HIST ? FU_WAVES * FU_HIST_SLOTS : 1];
    if (HIST) {
        for (int j = threadIdx.x; j < FU_WAVES * FU_HIST_SLOTS; j += FU_BLOCK) hist_all[j] = 0u;
    }
    const int copies = FU_HIST_SLOTS / K > 32 ? 32 : FU_HIST_SLOTS / K;
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    const int64_t *code_seg_off = LAYERS ? co3_cache_segs(code_seg_off_g, ncodes, code_seg_cache) : nullptr;
    // users and ranges in the reverse of the anchor pass's order: what that pass left in the last-level
    // cache is read first
    const int u = gridDim.y - 1 - blockIdx.y;
    const int64_t range = gridDim.x - 1 - blockIdx.x;
    if (!LAYERS) enc_all[threadIdx.x] = (int)threadIdx.x < K ? fcode_of(codes, u)->enc[threadIdx.x] : 0ull;
    __syncthreads();
    uint64_t *enc_s = LAYERS ? enc_all + (threadIdx.x / CO3_WAVE) * 256 : enc_all;
    int cur_code = -1;                   // LAYERS: the code whose table the wavefront holds

    const float *gu = g + (int64_t)u * stride;
    float *eu = err + (int64_t)u * stride;
    const int32_t *anchor_u = anchor + (int64_t)u * nseg;
    const float *scale_u = SCALED ? scale + (int64_t)u * nseg : nullptr;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    unsigned long long *stage = stage_all[wave];
    uint64_t *slots_u = slots + (int64_t)u * nunits * CO3_FUSED_SLOT_WORDS;
    uint32_t *unit_bits_u = unit_bits + (int64_t)u * nunits;
    uint32_t *chunk_local_u = chunk_local + (int64_t)u * nchunks;
    bool nocode = false;

    const int64_t beg = range * per_block;                               // a multiple of FU_TILE
    const int64_t end = beg + per_block < n ? beg + per_block : n;
    for (int64_t t0 = beg; t0 < end; t0 += FU_TILE) {
        const int64_t unit = t0 / CO3_FUSED_UNIT + wave;
        const int64_t u0 = unit * CO3_FUSED_UNIT;                         // first element of the wavefront's unit
        if (u0 >= n) continue;                                            // uniform over the wavefront
        const bool whole = u0 + CO3_FUSED_UNIT <= n;                      // uniform
        // anchor: one tensor for the whole unit (the usual case), else looked up per element
        const int64_t u_last = (whole ? u0 + CO3_FUSED_UNIT : n) - 1;
        const int s_lo = co3_find_seg(seg_off, nseg, u0), s_hi = co3_find_seg(seg_off, nseg, u_last);
        uint64_t acc[FU_SUB];            // the lane's four codewords of a run, joined (whole if they fit 64 bits)
        uint32_t qpack[FU_SUB];          // the four symbols of a run (looked up again if they do not)
        uint32_t nb[FU_SUB];             // bits of the lane's four codewords of a run
        bool one_code = true;
        if (LAYERS) {                    // the table of the unit's first element, reloaded when it changes
            const int c_lo = co3_find_seg(code_seg_off, ncodes, u0), c_hi = co3_find_seg(code_seg_off, ncodes, u_last);
            one_code = c_lo == c_hi;
            if (c_lo != cur_code) {      // uniform
                co3_wave_lds_sync();
                if (HIST && cur_code >= 0) flush_wave_counts(hist_all + wave * FU_HIST_SLOTS, copies, K, lane,
                                                             counts + (int64_t)cur_code * K);
                const Co3Code *cd = fcode_of(codes, c_lo);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int q = lane + k * CO3_WAVE;
                    enc_s[q] = q < K ? cd->enc[q] : 0ull;
                }
                co3_wave_lds_sync();
                cur_code = c_lo;
            }
        }
        const FusedUnit ua = {gu, eu, n, u0, lane, seg_off, nseg, anchor_u, scale_u, anchor_u[s_lo],
                                 SCALED ? scale_u[s_lo] : 1.0f, gamma, E, M, F, K, codemax, enc_s, codes, code_seg_off,
                                 ncodes, one_code, hist_all + wave * FU_HIST_SLOTS, copies, lane & (copies - 1), counts};
        if (whole && s_lo == s_hi && one_code) nocode |= fused_convert_unit<true, true, LAYERS, SCALED, HIST>(ua, acc, qpack, nb);
        else if (whole) nocode |= fused_convert_unit<true, false, LAYERS, SCALED, HIST>(ua, acc, qpack, nb);
        else nocode |= fused_convert_unit<false, false, LAYERS, SCALED, HIST>(ua, acc, qpack, nb);
        // positions: one scan per pair of runs
        uint32_t pos[FU_SUB], total = 0;
#pragma unroll
        for (int r = 0; r < FU_SUB; r += 2) {
            const uint32_t both = nb[r] | (nb[r + 1] << 16);
            const uint32_t incl = wave_scan_incl_u32(both, lane);
            const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, CO3_WAVE - 1);
            pos[r] = total + (incl & 0xffffu) - nb[r];
            total += tot & 0xffffu;
            pos[r + 1] = total + (incl >> 16) - nb[r + 1];
            total += tot >> 16;
        }
        // chunk index: position, inside the unit, of every chunk's first symbol (chunks start at multiples of 64)
#pragma unroll
        for (int r = 0; r < FU_SUB; ++r) {
            const int64_t i = u0 + r * FU_RUN + lane * FU_VEC;
            if (i < n && (i & (int64_t)(chunk_syms - 1)) == 0) chunk_local_u[i >> __builtin_ctz((unsigned)chunk_syms)] = pos[r];
        }

        // the unit's bits, packed from bit 0 of the wavefront's LDS window, then copied to the unit's slot
        const uint32_t nwords = (total + 63u) >> 6;                       // uniform; <= CO3_FUSED_SLOT_WORDS
        for (uint32_t w = lane; w <= nwords; w += CO3_WAVE) stage[w] = 0ull;    // one word of slack for the straddle test
        co3_wave_lds_sync();
#pragma unroll
        for (int r = 0; r < FU_SUB; ++r) {
            if (nb[r] <= 64u) {                      // the usual case: the lane's four codewords as one piece
                if (nb[r]) fused_stage(stage, acc[r], nb[r], pos[r]);
            } else {                                 // codeword by codeword, looked up again
                uint32_t p = pos[r];
#pragma unroll
                for (int k = 0; k < FU_VEC; ++k) {
                    const int64_t idx = u0 + r * FU_RUN + lane * FU_VEC + k;
                    const bool valid = whole || idx < n;
                    const uint64_t e = fused_entry<LAYERS>(ua, (qpack[r] >> (8 * k)) & 0xffu, valid ? idx : n - 1);
                    const uint32_t l = valid ? (uint32_t)(e & 63u) : 0u;
                    if (l) fused_stage(stage, e >> 6, l, p);
                    p += l;
                }
            }
        }
        co3_wave_lds_sync();
        uint64_t *slot = slots_u + unit * CO3_FUSED_SLOT_WORDS;
        for (uint32_t w = lane; w < nwords; w += CO3_WAVE) slot[w] = stage[w];
        if (lane == 0) unit_bits_u[unit] = total;
        co3_wave_lds_sync();                                              // the window is reused by the next unit
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
    if (HIST && LAYERS) {
        // the wavefronts of a block mostly end in the same code group: then one sum per block and symbol
        // (the pooled counters take an atomic from every block of every user)
        __shared__ int end_code[FU_WAVES];
        if (lane == 0) end_code[wave] = cur_code;
        __syncthreads();
        bool same = true;
        for (int w = 1; w < FU_WAVES; ++w) same &= end_code[w] == end_code[0];
        if (same) {
            if (end_code[0] >= 0) {
                for (int k = threadIdx.x; k < K; k += FU_BLOCK) {
                    uint32_t c = 0;
                    for (int w = 0; w < FU_WAVES; ++w)
                        for (int r = 0; r < copies; ++r) c += hist_all[w * FU_HIST_SLOTS + k * copies + r];
                    if (c) atomicAdd(&counts[(int64_t)end_code[0] * K + k], c);
                }
            }
        } else if (cur_code >= 0) {
            flush_wave_counts(hist_all + wave * FU_HIST_SLOTS, copies, K, lane, counts + (int64_t)cur_code * K);
        }
    } else if (HIST) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += FU_BLOCK) {
            uint32_t c = 0;
            for (int w = 0; w < FU_WAVES; ++w)
                for (int r = 0; r < copies; ++r) c += hist_all[w * FU_HIST_SLOTS + k * copies + r];
            if (c) atomicAdd(&counts[(int64_t)u * K + k], c);
        }
    }
}

// ---- pass 2: offsets of the units within groups of 64, group sizes -----------------------------
__global__ __launch_bounds__(CO3_WAVE) void k_unit_groups(const uint32_t *__restrict__ unit_bits,
                                                           uint32_t *__restrict__ unit_off,
                                                           uint64_t *__restrict__ groupsum, int64_t nunits, int64_t ngrp)
{
    const int u = blockIdx.y;
    const int64_t unit = (int64_t)blockIdx.x * CO3_FUSED_GROUP + threadIdx.x;
    const uint32_t size = unit < nunits ? unit_bits[(int64_t)u * nunits + unit] : 0u;
    const uint32_t incl = wave_scan_incl_u32(size, threadIdx.x);
    if (unit < nunits) unit_off[(int64_t)u * nunits + unit] = incl - size;
    if (threadIdx.x == CO3_WAVE - 1) groupsum[(int64_t)u * ngrp + blockIdx.x] = incl;
}

// ---- pass 4: every slot to its place in the stream; chunk index -------------------------------
// One wavefront per CP_UNITS consecutive units (all in one group of the scan).  Stream word gw belongs
// to the unit that holds its first bit; its content is 64 bits of the unit's slot from local bit
// 64*gw - D on (D = stream position of the unit), and where the unit ends inside the word, the leading
// bits of the next unit's slot.  The first 64 owned words of all units are loaded before any is stored.
#define CP_UNITS 4
#define CP_ROUNDS 2
static_assert(CO3_FUSED_GROUP % CP_UNITS == 0, "the units of a wavefront share a group");

__device__ __forceinline__ uint64_t compact_word(uint64_t s0, uint64_t s1, uint32_t sh, uint32_t a, uint32_t size,
                                                 uint64_t next0)
{
    uint64_t v = sh ? (s0 << sh) | (s1 >> (64u - sh)) : s0;
    const uint32_t rem = size - (a * 64u + sh);                          // bits of this unit from the word's first bit on
    if (rem < 64u) {                                                     // the unit ends inside this word
        v &= ~0ull << (64u - rem);
        v |= next0 >> rem;
    }
    return v;
}

__global__ __launch_bounds__(FU_BLOCK) void k_compact(const uint64_t *__restrict__ slots,
                                                       const uint32_t *__restrict__ unit_bits,
                                                       const uint32_t *__restrict__ unit_off,
                                                       const uint64_t *__restrict__ groupoff,
                                                       const uint32_t *__restrict__ chunk_local, int64_t n, int64_t nunits,
                                                       int64_t ngrp, uint64_t *__restrict__ words, int64_t cap_words,
                                                       int chunk_syms, uint64_t *__restrict__ chunk_bitoff, int64_t nchunks)
{
    const int u = blockIdx.y;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int64_t unit0 = ((int64_t)blockIdx.x * FU_WAVES + threadIdx.x / CO3_WAVE) * CP_UNITS;
    if (unit0 >= nunits) return;
    const uint32_t *bits_u = unit_bits + (int64_t)u * nunits;
    const uint32_t *off_u = unit_off + (int64_t)u * nunits;
    const uint64_t gbase = groupoff[(int64_t)u * ngrp + unit0 / CO3_FUSED_GROUP];
    // sizes of the wavefront's units and of the one after them (lane k holds unit0 + k), offsets likewise
    const bool have = lane <= CP_UNITS && unit0 + lane < nunits;
    const uint32_t my_size = have ? bits_u[unit0 + lane] : 0u;
    const uint32_t my_off = have ? off_u[unit0 + lane] : 0u;
    uint32_t size[CP_UNITS + 1], sh[CP_UNITS];
    uint64_t d[CP_UNITS];
#pragma unroll
    for (int k = 0; k <= CP_UNITS; ++k) size[k] = (uint32_t)__builtin_amdgcn_readlane((int)my_size, k);
#pragma unroll
    for (int k = 0; k < CP_UNITS; ++k) {
        d[k] = gbase + (uint32_t)__builtin_amdgcn_readlane((int)my_off, k);
        // every owned word of a unit starts at the same bit of a slot word (64 * gw - d is the same modulo
        // 64); the amount is uniform over the wavefront and is kept in a scalar register: an earlier build
        // that held it in the last vector register of the kernel's allocation produced wrong words in a few
        // wavefronts per thousand (cause not established), the scalar form never did
        sh[k] = (uint32_t)__builtin_amdgcn_readfirstlane((int)((0u - (uint32_t)d[k]) & 63u));
    }

    // chunk index: chunks whose first element lies in these units (chunks have at least 64 symbols)
    {
        const int64_t e0 = unit0 * CO3_FUSED_UNIT;
        const int64_t c = ((e0 + chunk_syms - 1) >> __builtin_ctz((unsigned)chunk_syms)) + lane;      // a power of two
        const int64_t e = c * chunk_syms;
        if (e < n && e < e0 + (int64_t)CP_UNITS * CO3_FUSED_UNIT) {
            const int k = (int)((e - e0) / CO3_FUSED_UNIT);
            uint64_t dk = d[0];
#pragma unroll
            for (int j = 1; j < CP_UNITS; ++j) dk = k == j ? d[j] : dk;
            chunk_bitoff[(int64_t)u * (nchunks + 1) + c] = dk + chunk_local[(int64_t)u * nchunks + c];
        }
    }
    static_assert(CP_UNITS * CO3_FUSED_UNIT / 64 <= CO3_WAVE, "one lane per possible chunk start");

    uint64_t *wu = words + (int64_t)u * cap_words;
    const uint64_t *slot0 = slots + ((int64_t)u * nunits + unit0) * CO3_FUSED_SLOT_WORDS;
    // the first CP_ROUNDS * 64 owned words of every unit are loaded before any is stored (two rounds cover
    // units of up to 8 bits per element); longer units finish in a loop
    uint64_t s0[CP_UNITS][CP_ROUNDS], s1[CP_UNITS][CP_ROUNDS], next0[CP_UNITS], gw0[CP_UNITS];
    uint32_t nown[CP_UNITS];
#pragma unroll
    for (int k = 0; k < CP_UNITS; ++k) {
        const uint64_t *slot = slot0 + (int64_t)k * CO3_FUSED_SLOT_WORDS;
        gw0[k] = (d[k] + 63) >> 6;                                       // owned words [gw0, gw0 + nown)
        const uint64_t gw1 = (d[k] + size[k] + 63) >> 6;
        // beyond the capacity nothing is written (the scan pass has reported it)
        nown[k] = size[k] == 0u || gw1 > (uint64_t)cap_words ? 0u : (uint32_t)(gw1 - gw0[k]);
        const uint32_t nw = (size[k] + 63u) >> 6;                        // words of the slot that hold bits
#pragma unroll
        for (int r = 0; r < CP_ROUNDS; ++r) {
            const uint32_t a = (uint32_t)lane + r * CO3_WAVE;
            s0[k][r] = a < nown[k] ? slot[a] : 0ull;
            s1[k][r] = a < nown[k] && a + 1u < nw ? slot[a + 1u] : 0ull;
        }
        next0[k] = nown[k] && size[k + 1] ? slot[CO3_FUSED_SLOT_WORDS] : 0ull;   // first word of the next unit's slot
    }
#pragma unroll
    for (int k = 0; k < CP_UNITS; ++k)
#pragma unroll
        for (int r = 0; r < CP_ROUNDS; ++r) {
            const uint32_t a = (uint32_t)lane + r * CO3_WAVE;
            if (a < nown[k]) wu[gw0[k] + a] = compact_word(s0[k][r], s1[k][r], sh[k], a, size[k], next0[k]);
        }
#pragma unroll
    for (int k = 0; k < CP_UNITS; ++k) {                                 // units of more words than that
        const uint64_t *slot = slot0 + (int64_t)k * CO3_FUSED_SLOT_WORDS;
        const uint32_t nw = (size[k] + 63u) >> 6;
        for (uint32_t a = lane + CP_ROUNDS * CO3_WAVE; a < nown[k]; a += CO3_WAVE)
            wu[gw0[k] + a] = compact_word(slot[a], a + 1u < nw ? slot[a + 1u] : 0ull, sh[k], a, size[k], next0[k]);
    }
}

// Workspace carve-up shared by the host-side size function and the launcher.
struct FusedWs {
    size_t slots, unit_bits, unit_off, groupsum, chunk_local, total;
};
static FusedWs fused_layout(int64_t n, int U, int chunk_syms)
{
    const size_t nunits = (size_t)((n + CO3_FUSED_UNIT - 1) / CO3_FUSED_UNIT > 0 ? (n + CO3_FUSED_UNIT - 1) / CO3_FUSED_UNIT : 1);
    const size_t ngrp = (nunits + CO3_FUSED_GROUP - 1) / CO3_FUSED_GROUP;
    const size_t nchunks = (size_t)((n + chunk_syms - 1) / chunk_syms > 0 ? (n + chunk_syms - 1) / chunk_syms : 1);
    auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
    FusedWs w;
    w.slots = 0;
    w.unit_bits = w.slots + up((size_t)U * nunits * CO3_FUSED_SLOT_WORDS * 8 + 8);   // + the word read past the last slot
    w.unit_off = w.unit_bits + up((size_t)U * nunits * 4);
    w.groupsum = w.unit_off + up((size_t)U * nunits * 4);
    w.chunk_local = w.groupsum + up((size_t)U * ngrp * 8);
    w.total = w.chunk_local + up((size_t)U * nchunks * 4);
    return w;
}

size_t co3_fused_workspace_bytes_impl(int64_t n, int U, int chunk_syms) { return fused_layout(n, U, chunk_syms).total; }

hipError_t co3_launch_convert_encode(const float *g, float *err, int64_t n, int U, int64_t stride, const int64_t *seg_off,
                                     int nseg, const int32_t *anchor, const float *scale, float gamma, co3_fmt fmt,
                                     const void *codes, const int64_t *code_seg_off, int ncodes, uint32_t *counts,
                                     uint64_t *words, int64_t cap_words, int chunk_syms, uint64_t *chunk_bitoff,
                                     uint64_t *total_bits, void *workspace, int32_t *status, hipStream_t st)
{
    const int64_t nunits = (n + CO3_FUSED_UNIT - 1) / CO3_FUSED_UNIT;
    const int64_t ngrp = (nunits + CO3_FUSED_GROUP - 1) / CO3_FUSED_GROUP;
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    const FusedWs L = fused_layout(n, U, chunk_syms);
    char *ws = static_cast<char *>(workspace);
    uint64_t *slots = reinterpret_cast<uint64_t *>(ws + L.slots);
    uint32_t *unit_bits = reinterpret_cast<uint32_t *>(ws + L.unit_bits);
    uint32_t *unit_off = reinterpret_cast<uint32_t *>(ws + L.unit_off);
    uint64_t *groupsum = reinterpret_cast<uint64_t *>(ws + L.groupsum);
    uint32_t *chunk_local = reinterpret_cast<uint32_t *>(ws + L.chunk_local);
    if (nunits > 0) {
        // about 2048 workgroups in all, each a whole number of block steps
        int64_t per_user = 2048 / U > 0 ? 2048 / U : 1;
        int64_t per_block = ((n + per_user - 1) / per_user + FU_TILE - 1) / FU_TILE * FU_TILE;
        const dim3 grid((unsigned)((n + per_block - 1) / per_block), U), block(FU_BLOCK);
        {
            Co3LaunchTimer tm(CO3_K_CONVERT, st);
#define CO3_STAGE_LAUNCH(L_, S_, H_)                                                                                    \
    hipLaunchKernelGGL((k_convert_stage<L_, S_, H_>), grid, block, 0, st, g, err, n, stride, seg_off, nseg, anchor,      \
                       scale, gamma, fmt, codes, code_seg_off, ncodes, counts, slots, unit_bits, chunk_local,           \
                       chunk_syms, nchunks, nunits, per_block, status)
            if (code_seg_off && scale && counts) CO3_STAGE_LAUNCH(true, true, true);
            else if (code_seg_off && scale) CO3_STAGE_LAUNCH(true, true, false);
            else if (code_seg_off && counts) CO3_STAGE_LAUNCH(true, false, true);
            else if (code_seg_off) CO3_STAGE_LAUNCH(true, false, false);
            else if (counts) CO3_STAGE_LAUNCH(false, false, true);
            else CO3_STAGE_LAUNCH(false, false, false);
#undef CO3_STAGE_LAUNCH
        }
        {
            Co3LaunchTimer tm(CO3_K_ENC_SIZES, st);
            hipLaunchKernelGGL(k_unit_groups, dim3((unsigned)ngrp, U), dim3(CO3_WAVE), 0, st, unit_bits, unit_off, groupsum,
                               nunits, ngrp);
        }
    }
    hipError_t e = co3_launch_enc_scan(groupsum, ngrp, U, cap_words, chunk_bitoff, nchunks, total_bits, status, st);
    if (e != hipSuccess) return e;
    if (nunits > 0) {
        Co3LaunchTimer tm(CO3_K_ENC_PACK, st);
        const int64_t per_block = (int64_t)FU_WAVES * CP_UNITS;
        hipLaunchKernelGGL(k_compact, dim3((unsigned)((nunits + per_block - 1) / per_block), U), dim3(FU_BLOCK), 0, st,
                           (const uint64_t *)slots, (const uint32_t *)unit_bits, (const uint32_t *)unit_off,
                           (const uint64_t *)groupsum, (const uint32_t *)chunk_local, n, nunits, ngrp, words, cap_words,
                           chunk_syms, chunk_bitoff, nchunks);
    }
    return hipGetLastError();
}
