// Compression h_Hf (Algorithm 1, user side): coded size of every tile of 1024 symbols, exclusive scan
// of the tile sizes per user, then bit packing.  In the packing pass one wavefront owns one tile (16
// symbols per lane): it looks the codewords up, scans the lengths, packs its bits in an LDS staging
// window and writes every 64-bit word whose first bit lies inside the tile -- completing the last
// such word with the leading codewords of the following symbols, so that each word of the stream is
// written exactly once, by one wavefront, with plain coalesced stores.
#include "co3_dev.h"
#include "kernels.h"

#include <atomic>

#define EN_BLOCK 256
#define EN_WAVES (EN_BLOCK / CO3_WAVE)
#define EN_LSYM 16                             // symbols per lane
#define EN_STAGE_WORDS 128                     // staging window: 8192 bits = 8 bits/symbol on average
static_assert(CO3_WAVE * EN_LSYM == CO3_PACK_SYMS, "tile geometry");

__device__ __forceinline__ const Co3Code *code_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// Eight symbols stored two per byte (the earlier one in the low half) -> two words of four symbol bytes.
__device__ __forceinline__ void unpack_nib8(uint32_t w, uint32_t &b0, uint32_t &b1)
{
    const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;      // symbols 0 2 4 6 / 1 3 5 7, one per byte
    b0 = (lo & 0xffu) | ((hi & 0xffu) << 8) | ((lo & 0xff00u) << 8) | ((hi & 0xff00u) << 16);
    b1 = ((lo >> 16) & 0xffu) | (((hi >> 16) & 0xffu) << 8) | ((lo >> 24) << 16) | ((hi >> 24) << 24);
}

// The 16 symbols from element i (a multiple of 16) on, all below n; NIB: the array holds two symbols per byte.
__device__ __forceinline__ void load_syms16_full(const uint8_t *su, int64_t i, bool nib, uint32_t s[4])
{
    if (nib) {
        const uint2 a = *reinterpret_cast<const uint2 *>(su + (i >> 1));
        unpack_nib8(a.x, s[0], s[1]);
        unpack_nib8(a.y, s[2], s[3]);
    } else {
        const uint4 a = *reinterpret_cast<const uint4 *>(su + i);
        s[0] = a.x; s[1] = a.y; s[2] = a.z; s[3] = a.w;
    }
}

__device__ __forceinline__ uint32_t load_sym1(const uint8_t *su, int64_t j, bool nib)
{
    return nib ? ((uint32_t)su[j >> 1] >> (4 * (int)(j & 1))) & 0xfu : (uint32_t)su[j];
}

// Loads the 16 symbols of this lane into s[0..4) (4 per word, first symbol in the low byte);
// returns how many lie below n.
__device__ __forceinline__ int load_syms16(const uint8_t *su, int64_t i, int64_t n, uint32_t s[4], bool nib = false)
{
    if (i + EN_LSYM <= n) {
        load_syms16_full(su, i, nib, s);
        return EN_LSYM;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) s[k] = 0;
    int c = 0;
    for (int64_t j = i; j < n; ++j, ++c) s[c >> 2] |= load_sym1(su, j, nib) << (8 * (c & 3));
    return c;
}

__device__ __forceinline__ void wave_lds_sync() { co3_wave_lds_sync(); }

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += (uint64_t)__shfl_xor((long long)v, o, CO3_WAVE);
    return v;
}

// ---- pass 1: coded size of every tile; a wavefront takes 4 consecutive tiles with all loads in
// flight before the first table lookup.  The 16 tiles of a workgroup form a group: the kernel
// leaves each tile's offset within its group in tilesum[] and the group's size in groupsum[], so
// the serial scan of pass 2 runs over 16 times fewer entries. ------------------------------------
#define SZ_TILES 4
#define SZ_GROUP (EN_WAVES * SZ_TILES)        // tiles per workgroup = CO3_PACK_GROUP

__global__ __launch_bounds__(EN_BLOCK) void k_enc_sizes(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                         const void *__restrict__ codes, int K,
                                                         uint64_t *__restrict__ tilesum, int64_t nblk,
                                                         uint64_t *__restrict__ groupsum, int64_t ngrp,
                                                         int32_t *status, int sym_nib)
{
    const int u = blockIdx.y;
    const Co3Code *cd = code_of(codes, u);
    __shared__ uint8_t len_s[256];
    __shared__ uint8_t pairlen_s[256];     // symbols two per byte: both lengths together, bit 7 set when one of them is 0
    __shared__ uint32_t tile_bits[SZ_GROUP];
    len_s[threadIdx.x] = (int)threadIdx.x < K ? cd->len[threadIdx.x] : (uint8_t)0;
    if (threadIdx.x < SZ_GROUP) tile_bits[threadIdx.x] = 0;
    if (sym_nib) {
        const int lo = threadIdx.x & 15, hi = threadIdx.x >> 4;
        const uint32_t l0 = lo < K ? cd->len[lo] : 0u, l1 = hi < K ? cd->len[hi] : 0u;
        pairlen_s[threadIdx.x] = (uint8_t)((l0 + l1) | (l0 == 0u || l1 == 0u ? 0x80u : 0u));
    }
    __syncthreads();

    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    const int64_t tb0 = ((int64_t)blockIdx.x * EN_WAVES + wave) * SZ_TILES;
    const bool nib = sym_nib != 0;
    const uint8_t *su = sym + (int64_t)u * (nib ? stride / 2 : stride);
    uint32_t s[SZ_TILES][4];
    bool nocode = false;
    if (tb0 >= nblk) {                                // uniform: nothing for this wavefront
    } else if (nib && (tb0 + SZ_TILES) * CO3_PACK_SYMS <= n) {     // uniform: four complete tiles, two symbols per byte
        uint2 raw[SZ_TILES];
#pragma unroll
        for (int t = 0; t < SZ_TILES; ++t)
            raw[t] = *reinterpret_cast<const uint2 *>(su + (((tb0 + t) * CO3_PACK_SYMS + (int64_t)lane * EN_LSYM) >> 1));
#pragma unroll
        for (int t = 0; t < SZ_TILES; ++t) {
            uint32_t bits = 0, flags = 0;    // one lookup per byte
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint32_t e = pairlen_s[((c < 4 ? raw[t].x : raw[t].y) >> (8 * (c & 3))) & 0xffu];
                bits += e & 0x7fu;
                flags |= e;
            }
            nocode |= (flags & 0x80u) != 0u;
            bits = wave_sum_u32(bits);
            if (lane == 0) tile_bits[wave * SZ_TILES + t] = bits;
        }
    } else if ((tb0 + SZ_TILES) * CO3_PACK_SYMS <= n) {     // uniform: all four tiles are complete
#pragma unroll
        for (int t = 0; t < SZ_TILES; ++t) {
            // ordinary (cached) loads: the packing pass reads the same symbols next
            load_syms16_full(su, (tb0 + t) * CO3_PACK_SYMS + (int64_t)lane * EN_LSYM, nib, s[t]);
        }
#pragma unroll
        for (int t = 0; t < SZ_TILES; ++t) {
            uint32_t bits = 0, minlen = 255u;
#pragma unroll
            for (int c = 0; c < EN_LSYM; ++c) {
                uint32_t l = len_s[(s[t][c >> 2] >> (8 * (c & 3))) & 0xffu];
                bits += l;
                minlen = min(minlen, l);
            }
            nocode |= minlen == 0u;
            bits = wave_sum_u32(bits);
            if (lane == 0) tile_bits[wave * SZ_TILES + t] = bits;
        }
    } else {                                          // the end of the vector
        for (int t = 0; t < SZ_TILES && tb0 + t < nblk; ++t) {
            const int64_t i = (tb0 + t) * CO3_PACK_SYMS + (int64_t)lane * EN_LSYM;
            const int nvalid = i < n ? load_syms16(su, i, n, s[0], nib) : 0;
            uint32_t bits = 0;
#pragma unroll
            for (int c = 0; c < EN_LSYM; ++c) {
                uint32_t l = len_s[(s[0][c >> 2] >> (8 * (c & 3))) & 0xffu];
                bits += c < nvalid ? l : 0u;
                nocode |= c < nvalid && l == 0u;
            }
            bits = wave_sum_u32(bits);
            if (lane == 0) tile_bits[wave * SZ_TILES + t] = bits;
        }
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
    __syncthreads();
    if (threadIdx.x < SZ_GROUP) {
        const int64_t tb = (int64_t)blockIdx.x * SZ_GROUP + threadIdx.x;
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int k = 0; k < SZ_GROUP; ++k) {
            const uint32_t b = tile_bits[k];
            before += k < (int)threadIdx.x ? b : 0u;
            all += b;
        }
        if (tb < nblk) tilesum[(int64_t)u * nblk + tb] = before;
        if (threadIdx.x == 0) groupsum[(int64_t)u * ngrp + blockIdx.x] = all;
    }
}

// The same pass for one code per tensor shared by all users (Sec. III (ii) as stated): a wavefront keeps
// the length table of the tensor it is in, reloading it when a tile lies in another tensor; symbols of
// a tile that straddles tensors read their lengths from the code blobs directly.
__global__ __launch_bounds__(EN_BLOCK) void k_enc_sizes_layers(const uint8_t *__restrict__ sym, int64_t n,
                                                                int64_t stride, const void *__restrict__ codes, int K,
                                                                const int64_t *__restrict__ seg_off_g, int nseg,
                                                                uint64_t *__restrict__ tilesum, int64_t nblk,
                                                                uint64_t *__restrict__ groupsum, int64_t ngrp,
                                                                int32_t *status)
{
    const int u = blockIdx.y;
    __shared__ uint32_t len_w[EN_WAVES][256 / 4];
    __shared__ uint32_t tile_bits[SZ_GROUP];
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    if (threadIdx.x < SZ_GROUP) tile_bits[threadIdx.x] = 0;
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    __syncthreads();

    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    const int64_t tb0 = ((int64_t)blockIdx.x * EN_WAVES + wave) * SZ_TILES;
    const uint8_t *su = sym + (int64_t)u * stride;
    const uint8_t *len_b = reinterpret_cast<const uint8_t *>(len_w[wave]);
    bool nocode = false;
    int cached = -1;
    for (int t = 0; t < SZ_TILES && tb0 + t < nblk; ++t) {
        const int64_t t_lo = (tb0 + t) * CO3_PACK_SYMS;
        const int64_t t_hi = (t_lo + CO3_PACK_SYMS < n ? t_lo + CO3_PACK_SYMS : n) - 1;
        const int s_lo = co3_find_seg(seg_off, nseg, t_lo), s_hi = co3_find_seg(seg_off, nseg, t_hi);
        const int64_t i = t_lo + (int64_t)lane * EN_LSYM;
        uint32_t s[4];
        const int nvalid = i < n ? load_syms16(su, i, n, s) : 0;
        uint32_t bits = 0;
        if (s_lo == s_hi) {              // uniform
            if (cached != s_lo) {
                wave_lds_sync();
                len_w[wave][lane] = reinterpret_cast<const uint32_t *>(code_of(codes, s_lo)->len)[lane];
                wave_lds_sync();
                cached = s_lo;
            }
#pragma unroll
            for (int c = 0; c < EN_LSYM; ++c) {
                const uint32_t sy = (s[c >> 2] >> (8 * (c & 3))) & 0xffu;
                const uint32_t l = (int)sy < K ? len_b[sy] : 0u;
                bits += c < nvalid ? l : 0u;
                nocode |= c < nvalid && l == 0u;
            }
        } else if (nvalid > 0) {
            // a tile that straddles tensors: lengths from the code blobs.  The lane's 16 symbols mostly lie in
            // one tensor: then one lookup of the tensor and 16 independent loads (a lookup and a load per
            // symbol in turn put 16 memory latencies into this wavefront, and the kernel ends with its
            // slowest one)
            const int c_first = co3_find_seg(seg_off, nseg, i), c_last = co3_find_seg(seg_off, nseg, i + nvalid - 1);
            const uint8_t *len_first = code_of(codes, c_first)->len;
#pragma unroll
            for (int c = 0; c < EN_LSYM; ++c) {
                const uint32_t sy = (s[c >> 2] >> (8 * (c & 3))) & 0xffu;
                const uint8_t *lp = c_first == c_last ? len_first
                                                      : code_of(codes, co3_find_seg(seg_off, nseg, c < nvalid ? i + c : i))->len;
                const uint32_t l = c < nvalid && (int)sy < K ? lp[sy] : 0u;
                bits += l;
                nocode |= c < nvalid && l == 0u;
            }
        }
        bits = wave_sum_u32(bits);
        if (lane == 0) tile_bits[wave * SZ_TILES + t] = bits;
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
    __syncthreads();
    if (threadIdx.x < SZ_GROUP) {
        const int64_t tb = (int64_t)blockIdx.x * SZ_GROUP + threadIdx.x;
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int k = 0; k < SZ_GROUP; ++k) {
            const uint32_t b = tile_bits[k];
            before += k < (int)threadIdx.x ? b : 0u;
            all += b;
        }
        if (tb < nblk) tilesum[(int64_t)u * nblk + tb] = before;
        if (threadIdx.x == 0) groupsum[(int64_t)u * ngrp + blockIdx.x] = all;
    }
}

// ---- pass 2: per user, exclusive scan of the group sizes (in place), stream length and capacity
// check --------------------------------------------------------------------------------------
#define SC_BLOCK 1024
#define SC_PER 8

__global__ __launch_bounds__(SC_BLOCK) void k_enc_scan(uint64_t *__restrict__ tilesum, int64_t nblk, int64_t cap_words,
                                                        uint64_t *__restrict__ chunk_bitoff, int64_t nchunks,
                                                        uint64_t *__restrict__ total_bits, int32_t *status)
{
    const int u = blockIdx.x;
    uint64_t *bs = tilesum + (int64_t)u * nblk;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    __shared__ uint64_t wave_tot[SC_BLOCK / CO3_WAVE];
    __shared__ uint64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();

    // the sizes of the next step are requested before the current step is scanned
    uint64_t nxt[SC_PER];
#pragma unroll
    for (int k = 0; k < SC_PER; ++k) {
        const int64_t i = (int64_t)threadIdx.x * SC_PER + k;
        nxt[k] = i < nblk ? bs[i] : 0;
    }
    for (int64_t base = 0; base < nblk; base += SC_BLOCK * SC_PER) {
        int64_t i0 = base + (int64_t)threadIdx.x * SC_PER;
        uint64_t v[SC_PER];
        uint64_t mine = 0;
#pragma unroll
        for (int k = 0; k < SC_PER; ++k) {
            v[k] = nxt[k];
            mine += v[k];
        }
#pragma unroll
        for (int k = 0; k < SC_PER; ++k) {
            const int64_t i = i0 + (int64_t)SC_BLOCK * SC_PER + k;
            nxt[k] = i < nblk ? bs[i] : 0;
        }
        uint64_t incl = mine;   // wave inclusive scan of 64-bit values
#pragma unroll
        for (int o = 1; o < CO3_WAVE; o <<= 1) {
            uint64_t t = (uint64_t)__shfl_up((long long)incl, o, CO3_WAVE);
            if (lane >= o) incl += t;
        }
        if (lane == CO3_WAVE - 1) wave_tot[wave] = incl;
        __syncthreads();
        uint64_t off = carry_s, tile_tot = 0;
        for (int w = 0; w < SC_BLOCK / CO3_WAVE; ++w) {
            uint64_t t = wave_tot[w];
            if (w < wave) off += t;
            tile_tot += t;
        }
        uint64_t running = off + incl - mine;
#pragma unroll
        for (int k = 0; k < SC_PER; ++k) {
            if (i0 + k < nblk) bs[i0 + k] = running;
            running += v[k];
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_s += tile_tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const uint64_t total = carry_s;
        total_bits[u] = total;
        chunk_bitoff[(int64_t)u * (nchunks + 1) + nchunks] = total;
        if ((total + 63) / 64 > (uint64_t)cap_words) co3_raise(status, CO3_ECAP);
    }
}

// ---- pass 3: bit packing ------------------------------------------------------------------
// Codewords of the lane's 16 symbols, concatenated four at a time.
// `entry(symbol, k)` returns the packed (codeword << 6 | length) of the lane's k-th symbol.
template <bool FULL, class Entry>
__device__ __forceinline__ void lookup_runs(Entry entry, const uint32_t s[4], int nvalid,
                                            uint64_t run[EN_LSYM / 4], uint32_t runbits[EN_LSYM / 4], uint32_t &mybits,
                                            bool &wide)
{
#pragma unroll
    for (int g = 0; g < EN_LSYM / 4; ++g) {
        uint64_t acc = 0;
        uint32_t nb = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint64_t e = (FULL || 4 * g + k < nvalid) ? entry((s[g] >> (8 * k)) & 0xffu, 4 * g + k) : 0ull;
            uint32_t l = (uint32_t)(e & 63u);
            acc = (acc << l) | (e >> 6);
            nb += l;
        }
        wide |= nb > 64u;
        run[g] = acc;
        runbits[g] = nb;
        mybits += nb;
    }
}

// The same for codes of at most 16 bits (then (codeword << 6 | length) sits in the low dword of a
// table entry and two codewords fit 32 bits): pairs are joined with 32-bit operations.
__device__ __forceinline__ void lookup_runs_short(const uint64_t *enc_s, const uint32_t s[4],
                                                  uint64_t run[EN_LSYM / 4], uint32_t runbits[EN_LSYM / 4],
                                                  uint32_t &mybits)
{
    const uint32_t *enc32 = reinterpret_cast<const uint32_t *>(enc_s);
#pragma unroll
    for (int g = 0; g < EN_LSYM / 4; ++g) {
        uint32_t e0 = enc32[2 * (s[g] & 0xffu)], e1 = enc32[2 * ((s[g] >> 8) & 0xffu)];
        uint32_t e2 = enc32[2 * ((s[g] >> 16) & 0xffu)], e3 = enc32[2 * (s[g] >> 24)];
        uint32_t l1 = e1 & 63u, l3 = e3 & 63u;
        uint32_t p01 = ((e0 >> 6) << l1) | (e1 >> 6);
        uint32_t p23 = ((e2 >> 6) << l3) | (e3 >> 6);
        uint32_t n23 = (e2 & 63u) + l3;
        uint32_t nb = (e0 & 63u) + l1 + n23;
        run[g] = ((uint64_t)p01 << n23) | (uint64_t)p23;
        runbits[g] = nb;
        mybits += nb;
    }
}

// Symbols stored two per byte (alphabets of at most 16 symbols: no codeword exceeds 15 bits): one lookup per
// byte in a table of codeword pairs, (both codewords joined << 6 | both lengths), the earlier symbol's
// codeword on top; the two pairs of four consecutive symbols make a run of at most 60 bits.
__device__ __forceinline__ void lookup_runs_pairs(const uint64_t *penc_s, uint2 raw, uint64_t run[EN_LSYM / 4],
                                                  uint32_t runbits[EN_LSYM / 4], uint32_t &mybits)
{
#pragma unroll
    for (int g = 0; g < EN_LSYM / 4; ++g) {
        const uint32_t w = (g < 2 ? raw.x : raw.y) >> (16 * (g & 1));
        const uint64_t p0 = penc_s[w & 0xffu], p1 = penc_s[(w >> 8) & 0xffu];
        const uint32_t l1 = (uint32_t)(p1 & 63u);
        const uint32_t nb = (uint32_t)(p0 & 63u) + l1;
        run[g] = ((p0 >> 6) << l1) | (p1 >> 6);
        runbits[g] = nb;
        mybits += nb;
    }
}

// ORs `nb` bits (right-aligned in `acc`, 1 <= nb <= 64) into the staging window at stream position
// `pos` (bits, relative to the first word of the tile); only words inside the window are touched.
__device__ __forceinline__ void stage_bits(unsigned long long *stage, int64_t win_w0, uint64_t acc, int nb,
                                           uint64_t pos)
{
    uint64_t v = acc << (64 - nb);
    int64_t w = (int64_t)(pos >> 6) - win_w0;
    int o = (int)(pos & 63);
    if (w >= 0 && w < EN_STAGE_WORDS) atomicOr(&stage[w], (unsigned long long)(v >> o));
    if (o + nb > 64 && w + 1 >= 0 && w + 1 < EN_STAGE_WORDS) atomicOr(&stage[w + 1], (unsigned long long)(v << (64 - o)));
}

// LAYERS = false: one code per user (codes[u]), its table shared by the workgroup.  LAYERS = true: one
// code per tensor shared by all users (codes[tensor]); each wavefront keeps the table of its tile's
// tensor, and a tile that straddles tensors (look-ahead included) reads its entries from the code
// blobs, tensor by element.
// The per-user form is compiled for eight wavefronts per SIMD (64 registers; a few spills on the rarely taken
// paths): the kernel is bound by the latency of its per-tile chain, and residency is what hides it (C3:
// 61 -> 55 us against six wavefronts per SIMD).
template <bool LAYERS>
__global__ __launch_bounds__(EN_BLOCK) __attribute__((amdgpu_waves_per_eu(LAYERS ? 5 : 8, LAYERS ? 5 : 8)))
void k_enc_pack(const uint8_t *__restrict__ sym, int64_t n, int64_t stride, const void *__restrict__ codes, int K,
                const int64_t *__restrict__ seg_off_g, int nseg, const uint64_t *__restrict__ tileoff, int64_t nblk,
                const uint64_t *__restrict__ groupoff, int64_t ngrp, uint64_t *__restrict__ words, int64_t cap_words,
                int chunk_syms, uint64_t *__restrict__ chunk_bitoff, int64_t nchunks, int sym_nib)
{
    const int u = blockIdx.y;
    const bool nib = !LAYERS && sym_nib != 0;
    __shared__ uint64_t enc_all[LAYERS ? EN_WAVES * 256 : 256];
    __shared__ uint64_t penc_s[LAYERS ? 1 : 256];        // codeword pairs, symbols two per byte
    __shared__ unsigned long long stage_all[EN_WAVES][EN_STAGE_WORDS];
    __shared__ int64_t seg_cache[LAYERS ? CO3_SEG_CACHE : 1];
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    const int64_t tb = (int64_t)blockIdx.x * EN_WAVES + wave;      // the wavefront's tile: elements [t0, t1)
    const int64_t t0 = tb * CO3_PACK_SYMS;
    const int64_t t1 = t0 + CO3_PACK_SYMS < n ? t0 + CO3_PACK_SYMS : n;
    const bool whole_tile = t1 - t0 == CO3_PACK_SYMS;
    // Everything the wavefront reads from memory apart from the tables is requested first, so that its latency
    // and that of the table load below (with its barrier) overlap.
    const uint8_t *su = sym + (int64_t)u * (nib ? stride / 2 : stride);
    uint64_t *wu = words + (int64_t)u * cap_words;
    const int64_t i = t0 + (int64_t)lane * EN_LSYM;
    const bool live = tb < nblk;                     // uniform: the wavefront has a tile
    // a complete tile of symbols stored two per byte stays in that form: one lookup per byte below
    const bool raw_tile = nib && whole_tile;
    uint32_t s[4] = {0u, 0u, 0u, 0u};
    uint2 raw = make_uint2(0u, 0u);
    int nvalid = EN_LSYM;
    if (raw_tile) raw = *reinterpret_cast<const uint2 *>(su + (i >> 1));
    else if (whole_tile) load_syms16_full(su, i, nib, s);
    else nvalid = live && i < t1 ? load_syms16(su, i, t1, s, nib) : 0;
    // the symbols that follow the tile (their codewords complete its last word): used at the end
    const int64_t i2 = t1 + lane;
    const bool has_next = live && t1 > t0 && lane < CO3_WAVE - 1 && i2 < n;
    const uint32_t next_sym = has_next ? load_sym1(su, i2, nib) : 0u;
    const uint64_t group_base = live ? groupoff[(int64_t)u * ngrp + tb / CO3_PACK_GROUP] : 0ull;
    const uint64_t tile_base = live ? tileoff[(int64_t)u * nblk + tb] : 0ull;

    const uint64_t *enc_s = LAYERS ? enc_all + wave * 256 : enc_all;
    const int64_t *seg_off = seg_off_g;
    uint32_t maxlen;
    bool one_tensor = true;
    if (!LAYERS) {
        const Co3Code *cd = code_of(codes, u);
        for (int j = threadIdx.x; j < 256; j += blockDim.x) {
            enc_all[j] = j < K ? cd->enc[j] : 0ull;
            if (nib) {
                const int lo = j & 15, hi = j >> 4;
                const uint64_t e0 = lo < K ? cd->enc[lo] : 0ull, e1 = hi < K ? cd->enc[hi] : 0ull;
                const uint32_t l1 = (uint32_t)(e1 & 63u);
                penc_s[j] = ((((e0 >> 6) << l1) | (e1 >> 6)) << 6) | (uint64_t)((uint32_t)(e0 & 63u) + l1);
            }
        }
        maxlen = cd->maxlen;
        __syncthreads();
        if (tb >= nblk) return;
    } else {
        seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
        __syncthreads();
        if (tb >= nblk) return;
        // tensors of the tile and of the at most 63 following symbols whose codewords complete its last word
        const int64_t t_lo = t0;
        int64_t t_hi = t_lo + CO3_PACK_SYMS + CO3_WAVE - 1;
        t_hi = (t_hi < n ? t_hi : n) - 1;
        const int s_lo = co3_find_seg(seg_off, nseg, t_lo), s_hi = co3_find_seg(seg_off, nseg, t_hi);
        one_tensor = s_lo == s_hi;
        maxlen = 64u;                    // a mixed tile takes the general path
        if (one_tensor) {
            const Co3Code *cd = code_of(codes, s_lo);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int q = lane + k * CO3_WAVE;
                enc_all[wave * 256 + q] = q < K ? cd->enc[q] : 0ull;
            }
            maxlen = cd->maxlen;
            wave_lds_sync();
        }
    }
    unsigned long long *stage = stage_all[wave];

    // packed (codeword << 6 | length) of symbol sy at element idx
    auto entry_at = [&](uint32_t sy, int64_t idx) -> uint64_t {
        if (!LAYERS || one_tensor) return enc_s[sy];
        return (int)sy < K ? code_of(codes, co3_find_seg(seg_off, nseg, idx))->enc[sy] : 0ull;
    };
    // the lane's own symbols in a tile that straddles tensors: mostly one tensor, looked up once, so that the
    // 16 reads from its code blob are independent
    int c_first = 0, c_last = 0;
    if (LAYERS && !one_tensor && nvalid > 0) {
        c_first = co3_find_seg(seg_off, nseg, i);
        c_last = co3_find_seg(seg_off, nseg, i + nvalid - 1);
    }
    const uint64_t *enc_first = LAYERS ? code_of(codes, c_first)->enc : nullptr;
    auto entry = [&](uint32_t sy, int k) -> uint64_t {
        if (!LAYERS || one_tensor) return enc_s[sy];
        if (c_first == c_last) return (int)sy < K ? enc_first[sy] : 0ull;
        return entry_at(sy, i + k);
    };

    // One table lookup per symbol: the codewords of every 4 symbols are concatenated into one run
    // (kept in registers) as long as the run fits 64 bits, which it always does for codes of at most
    // 16 bits; a lane that meets a longer run falls back to symbol-by-symbol packing below.
    uint64_t run[EN_LSYM / 4];
    uint32_t runbits[EN_LSYM / 4];
    uint32_t mybits = 0;
    bool wide = false;
    if (raw_tile) {
        lookup_runs_pairs(penc_s, raw, run, runbits, mybits);
    } else if (whole_tile) {    // uniform: every symbol of the tile exists
        if (maxlen <= 16u)
            lookup_runs_short(enc_s, s, run, runbits, mybits);
        else
            lookup_runs<true>(entry, s, nvalid, run, runbits, mybits, wide);
    } else
        lookup_runs<false>(entry, s, nvalid, run, runbits, mybits, wide);
    const uint32_t incl = wave_scan_incl_u32(mybits, lane);
    const uint32_t excl = incl - mybits;
    const uint32_t tilebits = (uint32_t)__builtin_amdgcn_readlane((int)incl, CO3_WAVE - 1);

    const uint64_t B0 = group_base + tile_base;
    const uint64_t B1 = B0 + tilebits;

    // chunk index: stream position of every chunk that starts at this lane's first symbol
    // (chunk sizes are powers of two: a shift, not a 64-bit division that every lane of the wavefront would sit through)
    if (nvalid > 0 && (i & (int64_t)(chunk_syms - 1)) == 0)
        chunk_bitoff[(int64_t)u * (nchunks + 1) + (i >> __builtin_ctz((unsigned)chunk_syms))] = B0 + excl;
    // beyond the capacity nothing is written (the scan pass has reported it); uniform over the wavefront
    if ((B1 + 63) / 64 > (uint64_t)cap_words || tilebits == 0) return;

    const int64_t gw0 = (int64_t)(B0 >> 6);          // first and last stream word the tile touches
    const int64_t gwl = (int64_t)((B1 - 1) >> 6);
    const int64_t first_owned = (B0 & 63) ? gw0 + 1 : gw0;   // words whose first bit lies in the tile
    const uint64_t rel0 = (B0 & 63) + excl;          // position of this lane's bits, relative to word gw0

    if ((B0 & 63) + tilebits <= EN_STAGE_WORDS * 64u && !__any(wide)) {
        // usual case: the tile fits one staging window and every run fits 64 bits
#pragma unroll
        for (int j = 0; j < EN_STAGE_WORDS / CO3_WAVE; ++j) stage[lane + j * CO3_WAVE] = 0ull;
        wave_lds_sync();
        uint32_t pos = (uint32_t)rel0;
#pragma unroll
        for (int g = 0; g < EN_LSYM / 4; ++g) {
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
        if (B1 & 63) {          // complete the last word with the codewords that follow the tile
            uint64_t e = has_next ? entry_at(next_sym, i2) : 0ull;
            uint32_t l = (uint32_t)(e & 63u);
            uint32_t o = wave_scan_incl_u32(l, lane) - l;
            const uint32_t used = (uint32_t)(B1 & 63);
            if (l && used + o < 64u)
                atomicOr(&stage[last_rel], (unsigned long long)(((e >> 6) << (64 - l)) >> (used + o)));
        }
        wave_lds_sync();
        const uint32_t first_rel = (uint32_t)(first_owned - gw0);
#pragma unroll
        for (int j = 0; j < EN_STAGE_WORDS / CO3_WAVE; ++j) {
            const uint32_t r = lane + j * CO3_WAVE;
            if (r >= first_rel && r <= last_rel) wu[gw0 + r] = stage[r];
        }
        return;
    }

    for (int64_t win_w0 = 0; gw0 + win_w0 <= gwl; win_w0 += EN_STAGE_WORDS) {
#pragma unroll
        for (int j = 0; j < EN_STAGE_WORDS / CO3_WAVE; ++j) stage[lane + j * CO3_WAVE] = 0ull;
        wave_lds_sync();
        if (!wide) {
            uint64_t pos = rel0;
#pragma unroll
            for (int g = 0; g < EN_LSYM / 4; ++g) {
                if (runbits[g]) stage_bits(stage, win_w0, run[g], (int)runbits[g], pos);
                pos += runbits[g];
            }
        } else {
            // runs of at most 64 bits, symbol by symbol
            uint64_t acc = 0, pos = rel0;
            int accbits = 0;
            for (int c = 0; c < nvalid; ++c) {
                uint64_t e = entry((s[c >> 2] >> (8 * (c & 3))) & 0xffu, c);
                int l = (int)(e & 63u);
                if (l) {
                    if (accbits + l > 64) {
                        stage_bits(stage, win_w0, acc, accbits, pos);
                        pos += accbits;
                        acc = 0;
                        accbits = 0;
                    }
                    acc = (acc << l) | (e >> 6);
                    accbits += l;
                }
            }
            if (accbits) stage_bits(stage, win_w0, acc, accbits, pos);
        }
        // The last word of the tile is completed with the first codewords of the symbols that follow
        // (at most 63 bits, hence at most 63 symbols), clipped at the word end.
        const int64_t last_rel = gwl - gw0 - win_w0;
        if ((B1 & 63) && last_rel >= 0 && last_rel < EN_STAGE_WORDS) {
            uint64_t e = has_next ? entry_at(next_sym, i2) : 0ull;
            uint32_t l = (uint32_t)(e & 63u);
            uint32_t o = wave_scan_incl_u32(l, lane) - l;
            const uint32_t used = (uint32_t)(B1 & 63);
            if (l && used + o < 64u)
                atomicOr(&stage[last_rel], (unsigned long long)(((e >> 6) << (64 - l)) >> (used + o)));
        }
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < EN_STAGE_WORDS / CO3_WAVE; ++j) {
            int64_t gw = gw0 + win_w0 + lane + j * CO3_WAVE;
            if (gw >= first_owned && gw <= gwl) wu[gw] = stage[lane + j * CO3_WAVE];
        }
        wave_lds_sync();
    }
}

hipError_t co3_launch_enc_scan(uint64_t *sizes, int64_t nsizes, int U, int64_t cap_words, uint64_t *chunk_bitoff,
                               int64_t nchunks, uint64_t *total_bits, int32_t *status, hipStream_t st)
{
    Co3LaunchTimer tm(CO3_K_ENC_SCAN, st);
    hipLaunchKernelGGL(k_enc_scan, dim3(U), dim3(SC_BLOCK), 0, st, sizes, nsizes, cap_words, chunk_bitoff, nchunks,
                       total_bits, status);
    return hipGetLastError();
}

// seg_off != NULL selects one code per tensor (codes[tensor], shared by the users) instead of codes[user]
hipError_t co3_launch_encode(const uint8_t *sym, int64_t n, int U, int64_t stride, const void *codes, int K,
                             const int64_t *seg_off, int nseg, uint64_t *words, int64_t cap_words, int chunk_syms,
                             uint64_t *chunk_bitoff, uint64_t *total_bits, uint64_t *tilesum, int32_t *status,
                             hipStream_t st, int sym_nib)
{
    if (sym_nib && (seg_off || K > 16)) return hipErrorInvalidValue;
    static_assert(SZ_GROUP == CO3_PACK_GROUP, "group size of the sizes pass");
    const int64_t nblk = (n + CO3_PACK_SYMS - 1) / CO3_PACK_SYMS;
    const int64_t ngrp = (nblk + CO3_PACK_GROUP - 1) / CO3_PACK_GROUP;
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    uint64_t *groupsum = tilesum + (int64_t)U * (nblk > 0 ? nblk : 1);     // workspace: [U][nblk] then [U][ngrp]
    if (nblk > 0) {
        Co3LaunchTimer tm(CO3_K_ENC_SIZES, st);
        if (seg_off)
            hipLaunchKernelGGL(k_enc_sizes_layers, dim3((unsigned)ngrp, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes,
                               K, seg_off, nseg, tilesum, nblk, groupsum, ngrp, status);
        else
            hipLaunchKernelGGL(k_enc_sizes, dim3((unsigned)ngrp, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, K,
                               tilesum, nblk, groupsum, ngrp, status, sym_nib);
    }
    if (co3_launch_enc_scan(groupsum, ngrp, U, cap_words, chunk_bitoff, nchunks, total_bits, status, st) != hipSuccess)
        return hipGetLastError();
    if (nblk > 0) {
        const unsigned gx = (unsigned)((nblk + EN_WAVES - 1) / EN_WAVES);
        Co3LaunchTimer tm(CO3_K_ENC_PACK, st);
        if (seg_off)
            hipLaunchKernelGGL(k_enc_pack<true>, dim3(gx, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, K, seg_off,
                               nseg, (const uint64_t *)tilesum, nblk, (const uint64_t *)groupsum, ngrp, words,
                               cap_words, chunk_syms, chunk_bitoff, nchunks, 0);
        else
            hipLaunchKernelGGL(k_enc_pack<false>, dim3(gx, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, K, seg_off,
                               nseg, (const uint64_t *)tilesum, nblk, (const uint64_t *)groupsum, ngrp, words,
                               cap_words, chunk_syms, chunk_bitoff, nchunks, sym_nib);
    }
    return hipGetLastError();
}

// ---- the encoder's workspace for callers that cannot allocate --------------------------------------
// A fixed array in the library's device image (every GPU that loads the library holds its own copy until
// the process ends).  On the host the array's name is only a handle: its device address is looked up once
// per device and kept; kernels and copies only ever see that address.
static __device__ __align__(256) unsigned char scratch[CO3_ENCODE_STATIC_WS_BYTES];

#define CO3_MAX_DEVICES 64
hipError_t co3_static_encode_workspace(void **ptr_out)
{
    static std::atomic<void *> ptr_of[CO3_MAX_DEVICES];      // zero-initialised: nothing looked up yet
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= CO3_MAX_DEVICES) return hipErrorInvalidDevice;
    void *p = ptr_of[dev].load(std::memory_order_acquire);
    if (!p) {
        // two threads may both look it up: they get the same address
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr_of[dev].store(p, std::memory_order_release);
    }
    *ptr_out = p;
    return hipSuccess;
}
