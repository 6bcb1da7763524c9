// Compression h_Hf (Algorithm 1, user side): bit lengths per tile of 2048 symbols, exclusive scan
// of the tile lengths per user, then bit packing through an LDS staging window with coalesced
// 64-bit stores.  One wavefront owns one tile (32 symbols per lane), so the two passes over the
// symbols need no workgroup barriers.
#include "co3_dev.h"
#include "kernels.h"

#define EN_BLOCK 256
#define EN_WAVES (EN_BLOCK / CO3_WAVE)
#define EN_LSYM 32                             // symbols per lane
#define EN_STAGE_WORDS 256                     // staging window: 16384 bits = 8 bits/symbol on average
static_assert(CO3_WAVE * EN_LSYM == CO3_PACK_SYMS, "tile geometry");

__device__ __forceinline__ const Co3Code *code_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// Loads the 32 symbols of this lane into s[0..8) (4 per word, first symbol in the low byte);
// returns how many lie below n.
__device__ __forceinline__ int load_syms32(const uint8_t *su, int64_t i, int64_t n, uint32_t s[8])
{
    if (i + EN_LSYM <= n) {
        uint4 a = *reinterpret_cast<const uint4 *>(su + i);
        uint4 b = *reinterpret_cast<const uint4 *>(su + i + 16);
        s[0] = a.x; s[1] = a.y; s[2] = a.z; s[3] = a.w;
        s[4] = b.x; s[5] = b.y; s[6] = b.z; s[7] = b.w;
        return EN_LSYM;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) s[k] = 0;
    int c = 0;
    for (int64_t j = i; j < n; ++j, ++c) s[c >> 2] |= (uint32_t)su[j] << (8 * (c & 3));
    return c;
}

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- pass 1: coded size of every tile of 2048 symbols --------------------------------------
__global__ __launch_bounds__(EN_BLOCK) void k_enc_sizes(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                         const void *__restrict__ codes, int K,
                                                         uint64_t *__restrict__ blocksum, int64_t nblk, int32_t *status)
{
    const int u = blockIdx.y;
    const Co3Code *cd = code_of(codes, u);
    __shared__ uint8_t len_s[256];
    len_s[threadIdx.x] = (int)threadIdx.x < K ? cd->len[threadIdx.x] : (uint8_t)0;
    __syncthreads();

    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int64_t tb = (int64_t)blockIdx.x * EN_WAVES + threadIdx.x / CO3_WAVE;
    if (tb >= nblk) return;
    const uint8_t *su = sym + (int64_t)u * stride;
    const int64_t i = tb * CO3_PACK_SYMS + (int64_t)lane * EN_LSYM;
    uint32_t s[8];
    const int nvalid = i < n ? load_syms32(su, i, n, s) : 0;
    uint32_t bits = 0;
    bool nocode = false;
#pragma unroll
    for (int c = 0; c < EN_LSYM; ++c) {
        uint32_t l = len_s[(s[c >> 2] >> (8 * (c & 3))) & 0xffu];
        if (c < nvalid) {
            bits += l;
            nocode |= (l == 0);
        }
    }
    if (nocode) co3_raise(status, CO3_ENOCODE);
    bits = wave_sum_u32(bits);
    if (lane == 0) blocksum[(int64_t)u * nblk + tb] = bits;
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

__global__ __launch_bounds__(EN_BLOCK) void k_enc_pack(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                        const void *__restrict__ codes, int K,
                                                        const uint64_t *__restrict__ blockoff, int64_t nblk,
                                                        uint64_t *__restrict__ words, int64_t cap_words, int chunk_syms,
                                                        uint64_t *__restrict__ chunk_bitoff, int64_t nchunks,
                                                        const uint64_t *__restrict__ total_bits)
{
    const int u = blockIdx.y;
    const Co3Code *cd = code_of(codes, u);
    __shared__ uint64_t enc_s[256];
    __shared__ unsigned long long stage_all[EN_WAVES][EN_STAGE_WORDS];
    enc_s[threadIdx.x] = (int)threadIdx.x < K ? cd->enc[threadIdx.x] : 0ull;
    __syncthreads();

    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    const int64_t tb = (int64_t)blockIdx.x * EN_WAVES + wave;
    if (tb >= nblk) return;
    unsigned long long *stage = stage_all[wave];

    const uint64_t total = total_bits[u];
    const bool fits = (total + 63) / 64 <= (uint64_t)cap_words;
    const uint64_t B0 = blockoff[(int64_t)u * nblk + tb];
    const uint8_t *su = sym + (int64_t)u * stride;
    uint64_t *wu = words + (int64_t)u * cap_words;
    const int64_t i = tb * CO3_PACK_SYMS + (int64_t)lane * EN_LSYM;
    uint32_t s[8];
    const int nvalid = i < n ? load_syms32(su, i, n, s) : 0;

    // One table lookup per symbol: the codewords of every 4 symbols are concatenated into one run
    // (kept in registers) as long as the run fits 64 bits, which it always does for codes of at most
    // 16 bits; a lane that meets a longer run falls back to symbol-by-symbol packing below.
    uint64_t run[EN_LSYM / 4];
    uint32_t runbits[EN_LSYM / 4];
    uint32_t mybits = 0;
    bool wide = false;
#pragma unroll
    for (int g = 0; g < EN_LSYM / 4; ++g) {
        uint64_t acc = 0;
        uint32_t nb = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint64_t e = (4 * g + k < nvalid) ? enc_s[(s[g] >> (8 * k)) & 0xffu] : 0ull;
            uint32_t l = (uint32_t)(e & 63u);
            acc = (acc << l) | (e >> 6);
            nb += l;
        }
        wide |= nb > 64u;
        run[g] = acc;
        runbits[g] = nb;
        mybits += nb;
    }
    const uint32_t incl = wave_scan_incl_u32(mybits, lane);
    const uint32_t excl = incl - mybits;
    const uint32_t tilebits = (uint32_t)__shfl((int)incl, CO3_WAVE - 1, CO3_WAVE);

    // chunk index: stream position of every chunk that starts at this lane's first symbol
    if (nvalid > 0 && (i & (int64_t)(chunk_syms - 1)) == 0)
        chunk_bitoff[(int64_t)u * (nchunks + 1) + i / chunk_syms] = B0 + excl;

    if (!fits || tilebits == 0) return;   // uniform over the wavefront

    const uint64_t B1 = B0 + tilebits;
    const int64_t gw0 = (int64_t)(B0 >> 6);          // first and last stream word of the tile
    const int64_t gwl = (int64_t)((B1 - 1) >> 6);
    const uint64_t rel0 = (B0 & 63) + excl;          // position of this lane's bits, relative to word gw0

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
                uint64_t e = enc_s[(s[c >> 2] >> (8 * (c & 3))) & 0xffu];
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
        wave_lds_sync();
#pragma unroll
        for (int j = 0; j < EN_STAGE_WORDS / CO3_WAVE; ++j) {
            int64_t gw = gw0 + win_w0 + lane + j * CO3_WAVE;
            if (gw <= gwl) {
                unsigned long long v = stage[lane + j * CO3_WAVE];
                bool shared_word = (gw == gw0 && (B0 & 63)) || (gw == gwl && (B1 & 63));
                if (shared_word)
                    atomicOr(reinterpret_cast<unsigned long long *>(wu + gw), v);
                else
                    wu[gw] = v;
            }
        }
        wave_lds_sync();
    }
}

hipError_t co3_launch_encode(const uint8_t *sym, int64_t n, int U, int64_t stride, const void *codes, int K,
                             uint64_t *words, int64_t cap_words, int chunk_syms, uint64_t *chunk_bitoff,
                             uint64_t *total_bits, uint64_t *blocksum, int32_t *status, hipStream_t st)
{
    const int64_t nblk = (n + CO3_PACK_SYMS - 1) / CO3_PACK_SYMS;
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    const unsigned grid_x = (unsigned)((nblk + EN_WAVES - 1) / EN_WAVES);
    if (nblk > 0) {
        Co3LaunchTimer tm(CO3_K_ENC_SIZES, st);
        hipLaunchKernelGGL(k_enc_sizes, dim3(grid_x, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, K, blocksum,
                           nblk, status);
    }
    {
        Co3LaunchTimer tm(CO3_K_ENC_SCAN, st);
        hipLaunchKernelGGL(k_enc_scan, dim3(U), dim3(SC_BLOCK), 0, st, blocksum, nblk, words, cap_words, chunk_bitoff,
                           nchunks, total_bits, status);
    }
    Co3LaunchTimer tm(CO3_K_ENC_PACK, st);
    if (nblk > 0)
        hipLaunchKernelGGL(k_enc_pack, dim3(grid_x, U), dim3(EN_BLOCK), 0, st, sym, n, stride, codes, K,
                           (const uint64_t *)blocksum, nblk, words, cap_words, chunk_syms, chunk_bitoff, nchunks,
                           (const uint64_t *)total_bits);
    return hipGetLastError();
}
