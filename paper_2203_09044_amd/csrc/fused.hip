// User side of Algorithm 1 in one pass over g and the memory, for codes that are known before the
// iteration starts (tables designed from a model, Sec. III (ii), or kept from an earlier iteration):
// error correction, fp conversion and compression without the symbol array in between.
//
// The stream position of a codeword depends on all symbols before it, so the pass cannot write the
// stream itself.  Each wavefront converts a unit of 256 consecutive elements (four per lane), packs the
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
#define FU_TILE (FU_BLOCK * FU_VEC)             // elements of one block step: four units, one per wavefront
static_assert(CO3_FUSED_UNIT == CO3_WAVE * FU_VEC, "unit geometry");
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

// ---- pass 1: conversion with error correction, codeword lookup, unit-local packing -----------
__global__ __launch_bounds__(FU_BLOCK) void k_convert_stage(const float *__restrict__ g, float *__restrict__ err,
                                                             int64_t n, int64_t stride,
                                                             const int64_t *__restrict__ seg_off_g, int nseg,
                                                             const int32_t *__restrict__ anchor, float gamma, co3_fmt fmt,
                                                             const void *__restrict__ codes,
                                                             uint64_t *__restrict__ slots, uint32_t *__restrict__ unit_bits,
                                                             uint32_t *__restrict__ chunk_local, int chunk_syms,
                                                             int64_t nchunks, int64_t nunits, int64_t per_block,
                                                             int32_t *status)
{
    const FmtC fc(fmt);
    const int E = fc.E, M = fc.M, F = fc.F, K = fc.K, codemax = fc.codemax;
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    __shared__ uint64_t enc_s[256];
    __shared__ unsigned long long stage_all[FU_WAVES][CO3_FUSED_SLOT_WORDS + 1];
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    const int u = blockIdx.y;
    const Co3Code *cd = fcode_of(codes, u);
    enc_s[threadIdx.x] = (int)threadIdx.x < K ? cd->enc[threadIdx.x] : 0ull;
    const bool short_code = cd->maxlen <= 16u;       // four codewords of a lane fit 64 bits
    __syncthreads();

    const float *gu = g + (int64_t)u * stride;
    float *eu = err + (int64_t)u * stride;
    const int32_t *anchor_u = anchor + (int64_t)u * nseg;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    unsigned long long *stage = stage_all[wave];
    uint64_t *slots_u = slots + (int64_t)u * nunits * CO3_FUSED_SLOT_WORDS;
    uint32_t *unit_bits_u = unit_bits + (int64_t)u * nunits;
    uint32_t *chunk_local_u = chunk_local + (int64_t)u * nchunks;
    bool nocode = false;

    const int64_t beg = (int64_t)blockIdx.x * per_block;                 // a multiple of FU_TILE
    const int64_t end = beg + per_block < n ? beg + per_block : n;
    for (int64_t t0 = beg; t0 < end; t0 += FU_TILE) {
        const int64_t unit = t0 / CO3_FUSED_UNIT + wave;
        const int64_t u0 = unit * CO3_FUSED_UNIT;                         // first element of the wavefront's unit
        if (u0 >= n) continue;                                            // uniform over the wavefront
        const int64_t i = u0 + (int64_t)lane * FU_VEC;
        const int64_t left = n - i;
        const int nvalid = left >= FU_VEC ? FU_VEC : (left > 0 ? (int)left : 0);
        float gv[FU_VEC], ev[FU_VEC];
        if (nvalid == FU_VEC) {
            const float4 a = ld_stream_f4(gu + i), b = ld_stream_f4(eu + i);
            gv[0] = a.x; gv[1] = a.y; gv[2] = a.z; gv[3] = a.w;
            ev[0] = b.x; ev[1] = b.y; ev[2] = b.z; ev[3] = b.w;
        } else {
#pragma unroll
            for (int k = 0; k < FU_VEC; ++k) {
                gv[k] = k < nvalid ? gu[i + k] : 0.0f;
                ev[k] = k < nvalid ? eu[i + k] : 0.0f;
            }
        }
        // anchor: one tensor for the whole unit (the usual case), else looked up per element
        const int64_t u_last = (u0 + CO3_FUSED_UNIT < n ? u0 + CO3_FUSED_UNIT : n) - 1;
        const int s_lo = co3_find_seg(seg_off, nseg, u0), s_hi = co3_find_seg(seg_off, nseg, u_last);
        uint64_t ent[FU_VEC];
        uint32_t nb = 0;
        float en[FU_VEC];
#pragma unroll
        for (int k = 0; k < FU_VEC; ++k) {
            const int sg = s_lo == s_hi ? s_lo : co3_find_seg(seg_off, nseg, i + k < n ? i + k : n - 1);
            const int A = anchor_u[sg];
            const float x = gv[k] + gamma * ev[k];       // no contraction (build flag): one rounding per operation
            uint32_t q;
            float v;
            co3_quantize(x, A - F + 1, A, E, M, codemax, q, v);
            en[k] = x - v;
            const uint64_t e = k < nvalid ? enc_s[q] : 0ull;
            nocode |= k < nvalid && (e & 63u) == 0u;
            ent[k] = e;
            nb += (uint32_t)(e & 63u);
        }
        if (nvalid == FU_VEC) {
            st_stream_f4(eu + i, make_float4(en[0], en[1], en[2], en[3]));
        } else {
#pragma unroll
            for (int k = 0; k < FU_VEC; ++k)
                if (k < nvalid) eu[i + k] = en[k];
        }
        const uint32_t incl = wave_scan_incl_u32(nb, lane);
        const uint32_t excl = incl - nb;
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, CO3_WAVE - 1);
        if (nvalid > 0 && (i & (int64_t)(chunk_syms - 1)) == 0) chunk_local_u[i / chunk_syms] = excl;

        // the unit's bits, packed from bit 0 of the wavefront's LDS window, then copied to the unit's slot
        const uint32_t nwords = (total + 63u) >> 6;                       // uniform; <= CO3_FUSED_SLOT_WORDS
        for (uint32_t w = lane; w <= nwords; w += CO3_WAVE) stage[w] = 0ull;    // one word of slack for the straddle test
        co3_wave_lds_sync();
        if (short_code) {
            uint64_t acc = 0;
#pragma unroll
            for (int k = 0; k < FU_VEC; ++k) acc = (acc << (ent[k] & 63u)) | (ent[k] >> 6);
            if (nb) fused_stage(stage, acc, nb, excl);
        } else {
            uint32_t pos = excl;
#pragma unroll
            for (int k = 0; k < FU_VEC; ++k) {
                const uint32_t l = (uint32_t)(ent[k] & 63u);
                if (l) fused_stage(stage, ent[k] >> 6, l, pos);
                pos += l;
            }
        }
        co3_wave_lds_sync();
        uint64_t *slot = slots_u + unit * CO3_FUSED_SLOT_WORDS;
        for (uint32_t w = lane; w < nwords; w += CO3_WAVE) slot[w] = stage[w];
        if (lane == 0) unit_bits_u[unit] = total;
        co3_wave_lds_sync();                                              // the window is reused by the next unit
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
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
// One wavefront per four consecutive units.  Stream word gw belongs to the unit that holds its first
// bit; its content is 64 bits of the unit's slot from local bit 64*gw - D on (D = stream position of
// the unit), and where the unit ends inside the word, the leading bits of the next unit's slot.
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
    const int64_t tile = (int64_t)blockIdx.x * FU_WAVES + threadIdx.x / CO3_WAVE;
    const int64_t unit0 = tile * 4;
    if (unit0 >= nunits) return;
    const uint64_t *slots_u = slots + (int64_t)u * nunits * CO3_FUSED_SLOT_WORDS;
    const uint32_t *bits_u = unit_bits + (int64_t)u * nunits;
    const uint32_t *off_u = unit_off + (int64_t)u * nunits;
    const uint64_t gbase = groupoff[(int64_t)u * ngrp + unit0 / CO3_FUSED_GROUP];    // the four units share a group
    uint64_t D[4];
    uint32_t size[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const bool have = unit0 + k < nunits;
        size[k] = have ? bits_u[unit0 + k] : 0u;
        D[k] = gbase + (have ? off_u[unit0 + k] : 0u);
    }
#pragma unroll
    for (int k = 1; k < 4; ++k)
        if (unit0 + k >= nunits) D[k] = D[k - 1] + size[k - 1];

    // chunk index: chunks whose first element lies in this tile (at most 16: chunks have at least 64 symbols)
    {
        const int64_t e0 = unit0 * CO3_FUSED_UNIT;
        const int64_t c0 = (e0 + chunk_syms - 1) / chunk_syms;
        const int64_t c = c0 + lane;
        const int64_t e = c * chunk_syms;
        if (e < n && e < e0 + 4 * CO3_FUSED_UNIT) {
            const int k = (int)((e - e0) / CO3_FUSED_UNIT);
            const uint64_t d = k == 0 ? D[0] : k == 1 ? D[1] : k == 2 ? D[2] : D[3];
            chunk_bitoff[(int64_t)u * (nchunks + 1) + c] = d + chunk_local[(int64_t)u * nchunks + c];
        }
    }
    // beyond the capacity nothing is written (the scan pass has reported it); uniform over the wavefront
    if ((D[3] + size[3] + 63) / 64 > (uint64_t)cap_words) return;
    uint64_t *wu = words + (int64_t)u * cap_words;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (size[k] == 0u) continue;                                     // uniform
        const uint64_t d = D[k];
        const uint64_t gw0 = (d + 63) >> 6, gw1 = (d + size[k] + 63) >> 6;     // owned words [gw0, gw1)
        const uint32_t nw = (size[k] + 63u) >> 6;                        // words of the slot that hold bits
        const uint64_t *slot = slots_u + (unit0 + k) * CO3_FUSED_SLOT_WORDS;
        const bool has_next = unit0 + k + 1 < nunits;
        const uint64_t next0 = has_next ? slot[CO3_FUSED_SLOT_WORDS] : 0ull;   // first word of the next unit's slot
        const bool next_empty = !has_next || bits_u[unit0 + k + 1] == 0u;
        // every owned word starts at the same bit of a slot word: 64 * gw - d is the same modulo 64
        const uint32_t sh = (uint32_t)__builtin_amdgcn_readfirstlane((int)((0u - (uint32_t)d) & 63u));
        for (uint64_t gw = gw0 + lane; gw < gw1; gw += CO3_WAVE) {
            const uint32_t l = (uint32_t)((gw << 6) - d);                // local bit of the word's first bit
            const uint32_t a = l >> 6;
            const uint64_t s0 = slot[a];
            const uint64_t s1 = slot[a + 1u < nw ? a + 1u : a];
            uint64_t v = sh ? (s0 << sh) | ((a + 1u < nw ? s1 : 0ull) >> (64u - sh)) : s0;
            const uint32_t rem = size[k] - l;                            // bits of this unit from l on
            if (rem < 64u) {                                             // the unit ends inside this word
                v &= ~0ull << (64u - rem);
                if (!next_empty) v |= next0 >> rem;
            }
            wu[gw] = v;
        }
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
                                     int nseg, const int32_t *anchor, float gamma, co3_fmt fmt, const void *codes,
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
        const unsigned gx = (unsigned)((n + per_block - 1) / per_block);
        {
            Co3LaunchTimer tm(CO3_K_CONVERT, st);
            hipLaunchKernelGGL(k_convert_stage, dim3(gx, U), dim3(FU_BLOCK), 0, st, g, err, n, stride, seg_off, nseg, anchor,
                               gamma, fmt, codes, slots, unit_bits, chunk_local, chunk_syms, nchunks, nunits, per_block,
                               status);
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
        const int64_t ntiles = (nunits + 3) / 4;
        Co3LaunchTimer tm(CO3_K_ENC_PACK, st);
        hipLaunchKernelGGL(k_compact, dim3((unsigned)((ntiles + FU_WAVES - 1) / FU_WAVES), U), dim3(FU_BLOCK), 0, st,
                           (const uint64_t *)slots, (const uint32_t *)unit_bits, (const uint32_t *)unit_off,
                           (const uint64_t *)groupsum, (const uint32_t *)chunk_local, n, nunits, ngrp, words, cap_words,
                           chunk_syms, chunk_bitoff, nchunks);
    }
    return hipGetLastError();
}
