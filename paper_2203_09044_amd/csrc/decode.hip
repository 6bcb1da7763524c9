// Parameter-server side of Algorithm 1: chunk-indexed Huffman decoding with an LDS lookup
// table (one lane per chunk), and the average of the reconstructed user gradients.
#include "co3_dev.h"
#include "kernels.h"

#define DE_BLOCK 256

__device__ __forceinline__ const Co3Code *dcode_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// The stream as 32-bit pieces in stream order: piece q holds stream bits [32q, 32q+32), first bit
// in its top bit.  In memory the words are little-endian u64, so piece q is 32-bit element q ^ 1.
struct BitReader {
    const uint32_t *w32;
    int64_t npieces;     // 2 * cap_words: reads beyond are zeros
    uint64_t buf;        // upcoming bits, left-justified
    int avail;           // valid bits in buf
    int64_t q;           // next piece to load

    __device__ __forceinline__ uint32_t piece(int64_t k) const { return (k >= 0 && k < npieces) ? w32[k ^ 1] : 0u; }
    __device__ __forceinline__ void seek(uint64_t p)
    {
        int64_t k = (int64_t)(p >> 5);
        int o = (int)(p & 31);
        buf = (((uint64_t)piece(k) << 32) | (uint64_t)piece(k + 1)) << o;
        avail = 64 - o;
        q = k + 2;
    }
    __device__ __forceinline__ uint64_t pos() const { return (uint64_t)(q << 5) - (uint64_t)avail; }
    __device__ __forceinline__ void refill()
    {
        if (avail <= 32) {
            buf |= (uint64_t)piece(q) << (32 - avail);
            avail += 32;
            ++q;
        }
    }
    // 64 stream bits starting at absolute position p
    __device__ __forceinline__ uint64_t peek64(uint64_t p) const
    {
        int64_t k = (int64_t)(p >> 5);
        int o = (int)(p & 31);
        uint64_t hi = ((uint64_t)piece(k) << 32) | (uint64_t)piece(k + 1);
        uint64_t lo = (uint64_t)piece(k + 2);
        return o ? ((hi << o) | (lo >> (32 - o))) : hi;
    }
};

struct DecTables {           // LDS-resident decoder tables of one user
    uint16_t lut[1 << CO3_LUT_BITS_MAX];
    uint64_t first_code[65];
    uint16_t count[66];
    uint16_t base[66];
    uint8_t sorted[256];
    uint32_t maxlen, lut_bits;
};

__device__ __forceinline__ void load_tables(DecTables &t, const Co3Code *cd)
{
    const uint32_t lb = cd->lut_bits > CO3_LUT_BITS_MAX ? CO3_LUT_BITS_MAX : cd->lut_bits;
    for (uint32_t i = threadIdx.x; i < (1u << lb); i += blockDim.x) t.lut[i] = cd->lut[i];
    for (int i = threadIdx.x; i < 65; i += blockDim.x) t.first_code[i] = cd->first_code[i];
    for (int i = threadIdx.x; i < 66; i += blockDim.x) {
        t.count[i] = cd->count[i];
        t.base[i] = cd->base[i];
    }
    for (int i = threadIdx.x; i < 256; i += blockDim.x) t.sorted[i] = cd->sorted[i];
    if (threadIdx.x == 0) {
        t.maxlen = cd->maxlen > 64 ? 64 : cd->maxlen;
        t.lut_bits = lb < 1 ? 1 : lb;
    }
}

// Canonical decoding of a codeword longer than the table prefix: the first length l whose l-bit
// prefix lies within that length's codeword range.  Returns the length, 0 if there is none.
__device__ __forceinline__ int decode_long(const DecTables &t, uint64_t window, uint32_t *sym)
{
    for (uint32_t l = t.lut_bits + 1; l <= t.maxlen; ++l) {
        uint64_t off = (window >> (64 - l)) - t.first_code[l];
        if (off < (uint64_t)t.count[l]) {
            *sym = t.sorted[(t.base[l] + (uint32_t)off) & 255u];
            return (int)l;
        }
    }
    return 0;
}

// One lane decodes the `nsym` symbols of one chunk and stores them at out[0..nsym).
__device__ __forceinline__ bool decode_chunk(const DecTables &t, BitReader &br, uint64_t p0, uint64_t p1, int nsym,
                                             uint8_t *out)
{
    bool ok = true;
    const int shift = 64 - (int)t.lut_bits;
    br.seek(p0);
    int i = 0;
    for (; i + 16 <= nsym; i += 16) {
        uint32_t w[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            uint32_t acc = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                br.refill();
                uint32_t e = t.lut[br.buf >> shift];
                int l = (int)(e >> 8);
                uint32_t s = e & 0xffu;
                if (l == 0) {                       // rare: longer than the table prefix
                    uint64_t p = br.pos();
                    l = decode_long(t, br.peek64(p), &s);
                    if (l == 0) { ok = false; l = 1; s = 0; }
                    br.seek(p + l);
                } else {
                    br.buf <<= l;
                    br.avail -= l;
                }
                acc |= s << (8 * b);
            }
            w[a] = acc;
        }
        *reinterpret_cast<uint4 *>(out + i) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (; i < nsym; ++i) {
        br.refill();
        uint32_t e = t.lut[br.buf >> shift];
        int l = (int)(e >> 8);
        uint32_t s = e & 0xffu;
        if (l == 0) {
            uint64_t p = br.pos();
            l = decode_long(t, br.peek64(p), &s);
            if (l == 0) { ok = false; l = 1; s = 0; }
            br.seek(p + l);
        } else {
            br.buf <<= l;
            br.avail -= l;
        }
        out[i] = (uint8_t)s;
    }
    return ok && br.pos() == p1;
}

__global__ __launch_bounds__(DE_BLOCK) void k_decode(const uint64_t *__restrict__ words, int64_t cap_words,
                                                      const uint64_t *__restrict__ chunk_bitoff, int chunk_syms,
                                                      int64_t nchunks, const void *__restrict__ codes, int64_t n,
                                                      uint8_t *__restrict__ sym_out, int64_t stride, int32_t *status)
{
    const int u = blockIdx.y;
    __shared__ DecTables t;
    load_tables(t, dcode_of(codes, u));
    __syncthreads();

    const int64_t c = (int64_t)blockIdx.x * DE_BLOCK + threadIdx.x;
    if (c >= nchunks) return;
    const uint64_t *off = chunk_bitoff + (int64_t)u * (nchunks + 1);
    BitReader br;
    br.w32 = reinterpret_cast<const uint32_t *>(words + (int64_t)u * cap_words);
    br.npieces = 2 * cap_words;
    int64_t first = c * chunk_syms;
    int nsym = (int)(n - first < chunk_syms ? n - first : chunk_syms);
    bool ok = decode_chunk(t, br, off[c], off[c + 1], nsym, sym_out + (int64_t)u * stride + first);
    if (!ok) co3_raise(status, CO3_EBADSTREAM);
}

// ---- average of the reconstructed gradients: users added in index order, one division -----
#define PS_BLOCK 256
#define PS_VEC 4
#define PS_TILE (PS_BLOCK * PS_VEC)

__global__ __launch_bounds__(PS_BLOCK) void k_ps_sum(const uint8_t *__restrict__ sym, int64_t n, int U, int64_t stride,
                                                      const int32_t *__restrict__ anchor,
                                                      const int64_t *__restrict__ seg_off, int nseg, co3_fmt fmt,
                                                      float *__restrict__ avg_out)
{
    const FmtC fc(fmt);
    const int EM = fc.E + fc.M, M = fc.M, F = fc.F;
    const uint32_t cmask = (uint32_t)fc.codemax;
    const float fU = (float)U;
    for (int64_t t0 = (int64_t)blockIdx.x * PS_TILE; t0 < n; t0 += (int64_t)gridDim.x * PS_TILE) {
        int64_t t1 = t0 + PS_TILE < n ? t0 + PS_TILE : n;
        int s_lo = co3_find_seg(seg_off, nseg, t0);
        int s_hi = co3_find_seg(seg_off, nseg, t1 - 1);
        int64_t i = t0 + (int64_t)threadIdx.x * PS_VEC;
        if (s_lo == s_hi && i + PS_VEC <= t1) {
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
            for (int u = 0; u < U; ++u) {
                const int e_min = anchor[(int64_t)u * nseg + s_lo] - F + 1;
                uint32_t q = *reinterpret_cast<const uint32_t *>(sym + (int64_t)u * stride + i);
                uint32_t q0 = q & 0xffu, q1 = (q >> 8) & 0xffu, q2 = (q >> 16) & 0xffu, q3 = q >> 24;
                float v0 = co3_code_value(q0 & cmask, e_min, M), v1 = co3_code_value(q1 & cmask, e_min, M);
                float v2 = co3_code_value(q2 & cmask, e_min, M), v3 = co3_code_value(q3 & cmask, e_min, M);
                a0 += __uint_as_float(__float_as_uint(v0) | ((q0 >> EM) << 31));
                a1 += __uint_as_float(__float_as_uint(v1) | ((q1 >> EM) << 31));
                a2 += __uint_as_float(__float_as_uint(v2) | ((q2 >> EM) << 31));
                a3 += __uint_as_float(__float_as_uint(v3) | ((q3 >> EM) << 31));
            }
            *reinterpret_cast<float4 *>(avg_out + i) = make_float4(a0 / fU, a1 / fU, a2 / fU, a3 / fU);
        } else {
            for (int64_t j = i; j < i + PS_VEC && j < t1; ++j) {
                int s = (s_lo == s_hi) ? s_lo : co3_find_seg(seg_off, nseg, j);
                float a = 0.f;
                for (int u = 0; u < U; ++u) {
                    const int e_min = anchor[(int64_t)u * nseg + s] - F + 1;
                    uint32_t q = sym[(int64_t)u * stride + j];
                    float v = co3_code_value(q & cmask, e_min, M);
                    a += __uint_as_float(__float_as_uint(v) | ((q >> EM) << 31));
                }
                avg_out[j] = a / fU;
            }
        }
    }
}

hipError_t co3_launch_decode(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int chunk_syms,
                             const void *codes, int64_t n, int U, uint8_t *sym_out, int64_t stride, int32_t *status,
                             hipStream_t st)
{
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    if (nchunks <= 0) return hipSuccess;
    unsigned blocks = (unsigned)((nchunks + DE_BLOCK - 1) / DE_BLOCK);
    hipLaunchKernelGGL(k_decode, dim3(blocks, U), dim3(DE_BLOCK), 0, st, words, cap_words, chunk_bitoff, chunk_syms,
                       nchunks, codes, n, sym_out, stride, status);
    return hipGetLastError();
}

hipError_t co3_launch_ps_sum(const uint8_t *sym, int64_t n, int U, int64_t stride, const int32_t *anchor,
                             const int64_t *seg_off, int nseg, co3_fmt fmt, float *avg_out, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t tiles = (n + PS_TILE - 1) / PS_TILE;
    unsigned blocks = (unsigned)(tiles < 4096 ? tiles : 4096);
    hipLaunchKernelGGL(k_ps_sum, dim3(blocks), dim3(PS_BLOCK), 0, st, sym, n, U, stride, anchor, seg_off, nseg, fmt,
                       avg_out);
    return hipGetLastError();
}
