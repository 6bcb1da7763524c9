// Compression h_Hf (Algorithm 1, user side): bit lengths per block of 2048 symbols, exclusive scan
// of the block lengths per user, then bit packing through an LDS staging window with coalesced
// 64-bit stores.
#include "co3_dev.h"
#include "kernels.h"

#define EN_BLOCK 256
#define EN_SPT 8                               // symbols per thread
#define EN_STAGE_WORDS 256                     // staging window: 16384 bits = 8 bits/symbol on average
static_assert(EN_BLOCK * EN_SPT == CO3_PACK_SYMS, "block geometry");

__device__ __forceinline__ const Co3Code *code_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// Loads the 8 symbols of this thread (zero-extended); *nvalid = how many lie below n.
__device__ __forceinline__ uint64_t load_syms8(const uint8_t *su, int64_t i, int64_t n, int *nvalid)
{
    if (i + EN_SPT <= n) {
        *nvalid = EN_SPT;
        return *reinterpret_cast<const uint64_t *>(su + i);
    }
    uint64_t v = 0;
    int c = 0;
    for (int64_t j = i; j < n; ++j, ++c) v |= (uint64_t)su[j] << (8 * c);
    *nvalid = c;
    return v;
}

// block-wide exclusive scan of one u32 per thread; returns the exclusive prefix, *total = block sum
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t *wave_tot /*[EN_BLOCK/64]*/, uint32_t *total)
{
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    uint32_t incl = wave_scan_incl_u32(v, lane);
    if (lane == CO3_WAVE - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < EN_BLOCK / CO3_WAVE; ++w) {
        uint32_t t = wave_tot[w];
        if (w < wave) off += t;
        tot += t;
    }
    *total = tot;
    return off + incl - v;
}

// ---- pass 1: coded size of every block of 2048 symbols ------------------------------------
__global__ __launch_bounds__(EN_BLOCK) void k_enc_sizes(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                         const void *__restrict__ codes, uint64_t *__restrict__ blocksum,
                                                         int64_t nblk, int32_t *status)
{
    const int u = blockIdx.y;
    const int64_t b = blockIdx.x;
    const Co3Code *cd = code_of(codes, u);
    __shared__ uint8_t len_s[256];
    __shared__ uint32_t wave_tot[EN_BLOCK / CO3_WAVE];
    len_s[threadIdx.x] = cd->len[threadIdx.x];
    __syncthreads();

    const uint8_t *su = sym + (int64_t)u * stride;
    int64_t i = b * CO3_PACK_SYMS + (int64_t)threadIdx.x * EN_SPT;
    int nvalid = 0;
    uint64_t s8 = i < n ? load_syms8(su, i, n, &nvalid) : 0;
    uint32_t bits = 0;
    bool nocode = false;
#pragma unroll
    for (int c = 0; c < EN_SPT; ++c) {
        uint32_t l = len_s[(s8 >> (8 * c)) & 0xffu];
        if (c < nvalid) {
            bits += l;
            nocode |= (l == 0);
        }
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
    bits = wave_sum_u32(bits);
    if ((threadIdx.x & (CO3_WAVE - 1)) == 0) wave_tot[threadIdx.x / CO3_WAVE] = bits;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t t = 0;
        for (int w = 0; w < EN_BLOCK / CO3_WAVE; ++w) t += wave_tot[w];
        blocksum[(int64_t)u * nblk + b] = t;
    }
}

// ---- pass 2: per user, exclusive scan of the block sizes (in place), stream length, capacity
// check, and zeroing of the words shared by two neighbouring blocks -------------------------
#define SC_BLOCK 1024
#define SC_PER 4

__global__ __launch_bounds__(SC_BLOCK) void k_enc_scan(uint64_t *__restrict__ blocksum, int64_t nblk,
                                                        uint64_t *__restrict__ words, int64_t cap_words,
                                                        uint64_t *__restrict__ chunk_bitoff, int64_t nchunks,
                                                        uint64_t *__restrict__ total_bits, int32_t *status)
{
    const int u = blockIdx.x;
    uint64_t *bs = blocksum + (int64_t)u * nblk;
    uint64_t *wu = words + (int64_t)u * cap_words;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    __shared__ uint64_t wave_tot[SC_BLOCK / CO3_WAVE];
    __shared__ uint64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();

    for (int64_t base = 0; base < nblk; base += SC_BLOCK * SC_PER) {
        int64_t i0 = base + (int64_t)threadIdx.x * SC_PER;
        uint64_t v[SC_PER];
        uint64_t mine = 0;
#pragma unroll
        for (int k = 0; k < SC_PER; ++k) {
            v[k] = (i0 + k < nblk) ? bs[i0 + k] : 0;
            mine += v[k];
        }
        // wave inclusive scan of 64-bit values
        uint64_t incl = mine;
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
        uint64_t run = off + incl - mine;
#pragma unroll
        for (int k = 0; k < SC_PER; ++k) {
            if (i0 + k < nblk) bs[i0 + k] = run;
            run += v[k];
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_s += tile_tot;
        __syncthreads();
    }
    const uint64_t total = carry_s;
    const bool fits = (total + 63) / 64 <= (uint64_t)cap_words;
    if (threadIdx.x == 0) {
        total_bits[u] = total;
        chunk_bitoff[(int64_t)u * (nchunks + 1) + nchunks] = total;
        if (!fits) co3_raise(status, CO3_ECAP);
    }
    if (fits) {
        // words that two blocks (or the last block and the padding) both touch are OR-ed into
        for (int64_t i = threadIdx.x; i <= nblk; i += SC_BLOCK) {
            uint64_t p = i < nblk ? bs[i] : total;
            if ((p & 63) && (int64_t)(p >> 6) < cap_words) wu[p >> 6] = 0;
        }
    }
}

// ---- pass 3: bit packing ------------------------------------------------------------------
// ORs `nb` bits (right-aligned in `acc`, 1 <= nb <= 64) into the staging window at stream position
// `pos` (bits, relative to the first word of the block); only words inside the window are touched.
__device__ __forceinline__ void stage_bits(unsigned long long *stage, int64_t win_w0, uint64_t acc, int nb,
                                           uint64_t pos)
{
    uint64_t v = acc << (64 - nb);
    int64_t w = (int64_t)(pos >> 6) - win_w0;
    int o = (int)(pos & 63);
    if (w >= 0 && w < EN_STAGE_WORDS) atomicOr(&stage[w], (unsigned long long)(v >> o));
    if (o + nb > 64 && w + 1 >= 0 && w + 1 < EN_STAGE_WORDS) atomicOr(&stage[w + 1], (unsigned long long)(v << (64 - o)));
}

__global__ __launch_bounds__(EN_BLOCK) void k_enc_pack(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                        const void *__restrict__ codes,
                                                        const uint64_t *__restrict__ blockoff, int64_t nblk,
                                                        uint64_t *__restrict__ words, int64_t cap_words, int chunk_syms,
                                                        uint64_t *__restrict__ chunk_bitoff, int64_t nchunks,
                                                        const uint64_t *__restrict__ total_bits)
{
    const int u = blockIdx.y;
    const int64_t b = blockIdx.x;
    const Co3Code *cd = code_of(codes, u);
    __shared__ uint64_t enc_s[256];
    __shared__ unsigned long long stage[EN_STAGE_WORDS];
    __shared__ uint32_t wave_tot[EN_BLOCK / CO3_WAVE];
    enc_s[threadIdx.x] = cd->enc[threadIdx.x];

    const uint64_t total = total_bits[u];
    const bool fits = (total + 63) / 64 <= (uint64_t)cap_words;
    const uint64_t B0 = blockoff[(int64_t)u * nblk + b];
    __syncthreads();

    const uint8_t *su = sym + (int64_t)u * stride;
    uint64_t *wu = words + (int64_t)u * cap_words;
    const int64_t i = b * CO3_PACK_SYMS + (int64_t)threadIdx.x * EN_SPT;
    int nvalid = 0;
    uint64_t s8 = i < n ? load_syms8(su, i, n, &nvalid) : 0;

    uint32_t mybits = 0;
#pragma unroll
    for (int c = 0; c < EN_SPT; ++c)
        if (c < nvalid) mybits += (uint32_t)(enc_s[(s8 >> (8 * c)) & 0xffu] & 63u);
    uint32_t blockbits;
    uint32_t excl = block_scan_excl(mybits, wave_tot, &blockbits);

    // chunk index: stream position of every chunk that starts in this block
    if (nvalid > 0 && (i & (int64_t)(chunk_syms - 1)) == 0)
        chunk_bitoff[(int64_t)u * (nchunks + 1) + i / chunk_syms] = B0 + excl;

    if (!fits || blockbits == 0) return;   // block-uniform

    const uint64_t B1 = B0 + blockbits;
    const int64_t gw0 = (int64_t)(B0 >> 6);          // first and last stream word of the block
    const int64_t gwl = (int64_t)((B1 - 1) >> 6);
    const uint64_t rel0 = (B0 & 63) + excl;          // position of this thread's bits, relative to word gw0

    for (int64_t win_w0 = 0; gw0 + win_w0 <= gwl; win_w0 += EN_STAGE_WORDS) {
        for (int j = threadIdx.x; j < EN_STAGE_WORDS; j += EN_BLOCK) stage[j] = 0ull;
        __syncthreads();
        // concatenate this thread's codewords into runs of at most 64 bits and OR them in
        uint64_t acc = 0, pos = rel0;
        int accbits = 0;
#pragma unroll
        for (int c = 0; c < EN_SPT; ++c) {
            if (c < nvalid) {
                uint64_t e = enc_s[(s8 >> (8 * c)) & 0xffu];
                int l = (int)(e & 63u);
                if (l) {
                    if (accbits + l > 64) {
                        stage_bits(stage, win_w0, acc, accbits, pos);
                        pos += accbits;
                        acc = 0;
                        accbits = 0;
                    }
                    acc = (l == 64 ? 0 : (acc << l)) | (e >> 6);
                    accbits += l;
                }
            }
        }
        if (accbits) stage_bits(stage, win_w0, acc, accbits, pos);
        __syncthreads();
        for (int j = threadIdx.x; j < EN_STAGE_WORDS; j += EN_BLOCK) {
            int64_t gw = gw0 + win_w0 + j;
            if (gw <= gwl) {
                unsigned long long v = stage[j];
                bool shared_word = (gw == gw0 && (B0 & 63)) || (gw == gwl && (B1 & 63));
                if (shared_word)
                    atomicOr(reinterpret_cast<unsigned long long *>(wu + gw), v);
                else
                    wu[gw] = v;
            }
        }
        __syncthreads();
    }
}

hipError_t co3_launch_encode(const uint8_t *sym, int64_t n, int U, int64_t stride, const void *codes, uint64_t *words,
                             int64_t cap_words, int chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits,
                             uint64_t *blocksum, int32_t *status, hipStream_t st)
{
    const int64_t nblk = (n + CO3_PACK_SYMS - 1) / CO3_PACK_SYMS;
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    if (nblk > 0) {
        Co3LaunchTimer tm(CO3_K_ENC_SIZES, st);
        hipLaunchKernelGGL(k_enc_sizes, dim3((unsigned)nblk, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, blocksum,
                           nblk, status);
    }
    {
        Co3LaunchTimer tm(CO3_K_ENC_SCAN, st);
        hipLaunchKernelGGL(k_enc_scan, dim3(U), dim3(SC_BLOCK), 0, st, blocksum, nblk, words, cap_words, chunk_bitoff,
                           nchunks, total_bits, status);
    }
    Co3LaunchTimer tm(CO3_K_ENC_PACK, st);
    if (nblk > 0)
        hipLaunchKernelGGL(k_enc_pack, dim3((unsigned)nblk, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes,
                           (const uint64_t *)blocksum, nblk, words, cap_words, chunk_syms, chunk_bitoff, nchunks,
                           (const uint64_t *)total_bits);
    return hipGetLastError();
}
