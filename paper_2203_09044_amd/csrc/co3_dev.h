// Shared device-side definitions of libco3 (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/co3.h"

#define CO3_WAVE 64
#define CO3_LUT_BITS_MAX 12
#define CO3_MAX_CODE_LEN 57     // (code << 6 | len) must fit 64 bits; u32 weights cannot reach it
#define CO3_PACK_SYMS 1024      // symbols per encoder tile (one wavefront, 16 per lane)
#define CO3_PACK_GROUP 16       // tiles whose sizes one workgroup of the sizes pass adds up
#define CO3_FUSED_UNIT 1024      // elements that one wavefront of the single-pass path converts and packs together
#define CO3_FUSED_SLOT_WORDS 1024 // 64-bit words of workspace per unit: room for 1024 codewords of any length
#define CO3_FUSED_GROUP 64       // units per group of the offset scan (= lanes of a wavefront)
#define CO3_COOP_KPT_MAX 22      // resident-grid user side: 16-byte pieces of a gradient that a lane keeps in registers
#define CO3_COOP_KPT_BIG 48      // the same with part of the pieces in LDS

// Per-user code blob.  Bytes 0..K-1 (len) are the public wire header; the rest is private.
struct Co3Code {
    uint8_t len[256];          // code length per symbol, 0 = no code
    uint64_t enc[256];         // (codeword << 6) | length
    uint64_t first_code[65];   // right-aligned first codeword of each length (canonical order)
    uint16_t count[66];        // number of codewords of each length
    uint16_t base[66];         // index into sorted[] of the first symbol of each length
    uint8_t sorted[256];       // symbols ordered by (length, symbol)
    uint32_t nact;             // symbols that have a code
    uint32_t maxlen;           // longest code length
    uint32_t lut_bits;         // decoder table is indexed by this many leading bits
    uint32_t reserved;
    uint16_t lut[1 << CO3_LUT_BITS_MAX];   // (length << 8) | symbol, 0 = longer than lut_bits or invalid
};
static_assert(sizeof(Co3Code) <= CO3_CODE_BYTES, "code blob size");

// Derived constants of a sign/exponent/mantissa format (Sec. III (i)).
struct FmtC {
    int E, M;
    int F;          // top exponent field, 2^E - 1
    int K;          // alphabet size
    int codemax;    // largest magnitude code, 2^(E+M) - 1
    __host__ __device__ FmtC(co3_fmt f)
        : E(f.exp_bits), M(f.mant_bits), F((1 << f.exp_bits) - 1), K(1 << (1 + f.exp_bits + f.mant_bits)),
          codemax((1 << (f.exp_bits + f.mant_bits)) - 1) {}
};

// Streaming (non-temporal) 16-byte accesses for data that is touched once per kernel.
typedef float co3_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t co3_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 ld_stream_f4(const float *p)
{
    co3_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const co3_f32x4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream_f4(float *p, float4 a)
{
    co3_f32x4 v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<co3_f32x4 *>(p));
}
__device__ __forceinline__ uint4 ld_stream_u4(const void *p)
{
    co3_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const co3_u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void co3_raise(int32_t *status, int32_t code)
{
    if (status) atomicMin(status, code);
}

// Number of k in [1, nseg] with seg_off[k] <= i, kept below nseg: the segment that holds element i.
__device__ __forceinline__ int co3_find_seg(const int64_t *seg_off, int nseg, int64_t i)
{
    if (seg_off == nullptr || nseg <= 1) return 0;
    int lo = 1, hi = nseg + 1;   // first k in [1, nseg] with seg_off[k] > i, or nseg + 1
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (seg_off[mid] <= i) lo = mid + 1; else hi = mid;
    }
    int s = lo - 1;
    return s > nseg - 1 ? nseg - 1 : s;
}

// Tensor boundaries are looked up once or twice per tile; a block keeps them in LDS when they fit
// (the lookups are chains of dependent loads).  Returns the pointer to search from then on.
#define CO3_SEG_CACHE 512
__device__ __forceinline__ const int64_t *co3_cache_segs(const int64_t *seg_off, int nseg, int64_t *cache)
{
    if (seg_off == nullptr || nseg <= 1 || nseg + 1 > CO3_SEG_CACHE) return seg_off;
    for (int k = threadIdx.x; k <= nseg; k += blockDim.x) cache[k] = seg_off[k];
    __syncthreads();
    return cache;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    // row shifts and row broadcasts as in the scan below; a lane without a source takes 0, the identity here
    auto step = [](uint32_t x, uint32_t y) { return x > y ? x : y; };
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));   // row_bcast:15 -> rows 1, 3
    v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));   // row_bcast:31 -> rows 2, 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, CO3_WAVE - 1);                        // the last lane holds the maximum
}

// Inclusive prefix sum across the 64 lanes of a wavefront with data-parallel-primitive moves:
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0/2 is added to row
// 1/3 and the last lane of the lower half to the upper half.  Lanes without a source add 0.
__device__ __forceinline__ uint32_t wave_scan_incl_u32(uint32_t v, int /*lane*/)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// sum over the wavefront, returned in every lane
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_scan_incl_u32(v, 0), CO3_WAVE - 1);
}

// Value of a magnitude code under e_min = A - F + 1 (Sec. III (i)): exponent field f >= 1 is
// (1 + m/2^M) * 2^(e_min + f - 1); field 0 is (m/2^M) * 2^e_min.
__device__ __forceinline__ float co3_code_value(uint32_t code, int e_min, int M)
{
    uint32_t f = code >> M;
    uint32_t nbits = (code << (23 - M)) + ((uint32_t)(e_min - 1 + 127) << 23);
    float sub = ldexpf((float)code, e_min - M);
    return f ? __uint_as_float(nbits) : sub;
}

// ------------------------------------------------------------------------------------------
// Q_A on one value (Sec. III (i), nearest level, ties to even, saturating), returning the symbol
// byte and its value.  All steps are exact: scaling by a power of two, rint, scaling back.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void co3_quantize(float x, int e_min, int A, int E, int M, int codemax, uint32_t &sym,
                                             float &val)
{
    uint32_t bits = __float_as_uint(x);
    uint32_t abits = bits & 0x7fffffffu;
    float a = __uint_as_float(abits);
    int ex = (int)(abits >> 23) - 127;          // fp32 subnormals read -127, below every e_min
    int e = ex > e_min ? ex : e_min;            // clamped exponent
    int qe = e - M;                             // exponent of the local quantum
    float t = ldexpf(a, -qe);                   // |x| in quanta: exact, < 2^(M+1) for finite x
    t = fminf(t, (float)(4 << M));              // Inf/NaN: keep the integer conversion defined
    float r = rintf(t);                         // ties to even
    int code = ((e - e_min) << M) + (int)r;     // a carry out of the mantissa lands in the next field
    float mag = ldexpf(r, qe);
    if (code > codemax) {                       // above the top binade
        code = codemax;
        mag = ldexpf((float)((2 << M) - 1), A - M);
    }
    uint32_t s = code ? (bits >> 31) : 0u;      // one zero only
    sym = (s << (E + M)) | (uint32_t)code;
    val = __uint_as_float(__float_as_uint(mag) | (s << 31));
}

// LDS written by some lanes of a wavefront is read by others.  The LDS operations of one wavefront are
// carried out in program order and its lanes run in lockstep, so all that is needed is that the earlier
// operations have been carried out (the LDS counter) and that the compiler keeps the order.  A fence, even
// at wavefront scope, would also wait for every global load and store in flight: in a streaming loop that
// drains the memory pipeline at every hand-over.
__device__ __forceinline__ void co3_wave_lds_sync()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    asm volatile("" ::: "memory");
}
