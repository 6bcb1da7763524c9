// User side of Algorithm 1: exponent anchor, error correction + fp conversion + memory update,
// symbol histogram.  Streaming kernels: every block owns a contiguous range of one user's vector.
#include "co3_dev.h"
#include "kernels.h"

#define CV_BLOCK 256
#define CV_VEC 4                       // elements per thread per step (one 16-byte load)
#define CV_TILE (CV_BLOCK * CV_VEC)    // elements per block step
#define HIST_SLOTS 1024                // LDS counters per wavefront

// ------------------------------------------------------------------------------------------
// initial values: anchors start at the lower clamp (so atomicMax applies it), counts at zero (or at one,
// where the counts are to give every symbol a codeword)
// ------------------------------------------------------------------------------------------
__global__ void k_fill_i32(int32_t *a, int64_t na, int32_t va, uint32_t *b, int64_t nb, uint32_t vb)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = i; j < na; j += step) a[j] = va;
    for (int64_t j = i; j < nb; j += step) b[j] = vb;
}

// ------------------------------------------------------------------------------------------
// anchor: A = floor(log2 max|g|) per (user, segment) = biased exponent of the largest magnitude
// minus 127, at most 127; the lower clamp comes from the initial value.
// ------------------------------------------------------------------------------------------
#define AM_UNROLL 8
#define AM_TILE (CV_TILE * AM_UNROLL)   // elements per block step: eight 16-byte loads in flight per thread
#define AM_PARTS 8                      // tensor parts of a straddling tile reduced per pair of block barriers

// Block-wide maximum of the magnitude bit patterns, then one atomic per block, fired without a result
// (reading the anchor first, to skip the atomic when it is already large enough, was measured slower:
// the line is contended while the blocks finish).  Called under block-uniform conditions.
__device__ __forceinline__ void absmax_flush(uint32_t m, int32_t *anchor_us, uint32_t *red)
{
    m = wave_max_u32(m);
    if ((threadIdx.x & (CO3_WAVE - 1)) == 0) red[threadIdx.x / CO3_WAVE] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t mm = red[0];
        for (int w = 1; w < CV_BLOCK / CO3_WAVE; ++w) mm = mm > red[w] ? mm : red[w];
        int cand = (int)(mm >> 23) - 127;
        if (cand > 127) cand = 127;
        atomicMax(anchor_us, cand);
    }
    __syncthreads();
}

__device__ __forceinline__ uint32_t absmax4(float4 v, uint32_t m)
{
    uint32_t a0 = __float_as_uint(v.x) & 0x7fffffffu, a1 = __float_as_uint(v.y) & 0x7fffffffu;
    uint32_t a2 = __float_as_uint(v.z) & 0x7fffffffu, a3 = __float_as_uint(v.w) & 0x7fffffffu;
    a0 = a0 > a1 ? a0 : a1;
    a2 = a2 > a3 ? a2 : a3;
    a0 = a0 > a2 ? a0 : a2;
    return m > a0 ? m : a0;
}

__global__ __launch_bounds__(CV_BLOCK) void k_absmax(const float *__restrict__ g, int64_t n, int64_t stride,
                                                      const int64_t *__restrict__ seg_off_g, int nseg,
                                                      int32_t *__restrict__ anchor, int64_t per_block)
{
    const int u = blockIdx.y;
    const float *gu = g + (int64_t)u * stride;
    int32_t *anchor_u = anchor + (int64_t)u * nseg;
    __shared__ uint32_t red[CV_BLOCK / CO3_WAVE];
    __shared__ uint32_t parts[CV_BLOCK / CO3_WAVE][AM_PARTS];
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    int64_t beg = (int64_t)blockIdx.x * per_block;
    int64_t end = beg + per_block < n ? beg + per_block : n;
    if (beg >= end) return;

    int cur_seg = co3_find_seg(seg_off, nseg, beg);
    uint32_t m = 0;
    for (int64_t t0 = beg; t0 < end; t0 += AM_TILE) {
        int64_t t1 = t0 + AM_TILE < end ? t0 + AM_TILE : end;
        int s_lo = co3_find_seg(seg_off, nseg, t0);
        int s_hi = co3_find_seg(seg_off, nseg, t1 - 1);
        int64_t i = t0 + (int64_t)threadIdx.x * CV_VEC;
        if (s_lo == s_hi) {
            if (s_lo != cur_seg) {       // block-uniform branch
                absmax_flush(m, anchor_u + cur_seg, red);
                m = 0;
                cur_seg = s_lo;
            }
            if (t1 - t0 == AM_TILE) {
                float4 v[AM_UNROLL];
                // ordinary (cached) loads: the conversion pass reads g again, last-read part first
#pragma unroll
                for (int k = 0; k < AM_UNROLL; ++k)
                    v[k] = *reinterpret_cast<const float4 *>(gu + i + (int64_t)k * CV_TILE);
#pragma unroll
                for (int k = 0; k < AM_UNROLL; ++k) m = absmax4(v[k], m);
            } else {
                for (int k = 0; k < AM_UNROLL; ++k) {
                    int64_t j0 = i + (int64_t)k * CV_TILE;
                    if (j0 + CV_VEC <= t1) {
                        m = absmax4(*reinterpret_cast<const float4 *>(gu + j0), m);
                    } else {
                        for (int64_t j = j0; j < t1; ++j) {
                            uint32_t a = __float_as_uint(gu[j]) & 0x7fffffffu;
                            m = m > a ? m : a;
                        }
                    }
                }
            }
        } else {
            // The tile straddles tensors.  Its elements are loaded once, all loads in flight together as in
            // the plain case (a loop per tensor part would put one memory latency per part into this block,
            // and the kernel ends with its slowest block); then the parts are reduced from registers, up
            // to AM_PARTS of them per pair of block barriers.
            absmax_flush(m, anchor_u + cur_seg, red);
            m = 0;
            uint32_t a[AM_UNROLL][CV_VEC];
#pragma unroll
            for (int k = 0; k < AM_UNROLL; ++k) {
                const int64_t j0 = i + (int64_t)k * CV_TILE;
                if (j0 + CV_VEC <= t1) {
                    const float4 v = *reinterpret_cast<const float4 *>(gu + j0);
                    a[k][0] = __float_as_uint(v.x); a[k][1] = __float_as_uint(v.y);
                    a[k][2] = __float_as_uint(v.z); a[k][3] = __float_as_uint(v.w);
                } else {
#pragma unroll
                    for (int c = 0; c < CV_VEC; ++c) a[k][c] = j0 + c < t1 ? __float_as_uint(gu[j0 + c]) : 0u;
                }
#pragma unroll
                for (int c = 0; c < CV_VEC; ++c) a[k][c] &= 0x7fffffffu;
            }
            for (int sg0 = s_lo; sg0 <= s_hi; sg0 += AM_PARTS) {
                const int np = s_hi - sg0 + 1 < AM_PARTS ? s_hi - sg0 + 1 : AM_PARTS;
                for (int p = 0; p < np; ++p) {
                    const int64_t a0 = seg_off[sg0 + p], a1 = seg_off[sg0 + p + 1];
                    uint32_t part = 0;
#pragma unroll
                    for (int k = 0; k < AM_UNROLL; ++k)
#pragma unroll
                        for (int c = 0; c < CV_VEC; ++c) {
                            const int64_t j = i + (int64_t)k * CV_TILE + c;
                            const uint32_t v = j >= a0 && j < a1 ? a[k][c] : 0u;
                            part = part > v ? part : v;
                        }
                    part = wave_max_u32(part);
                    if ((threadIdx.x & (CO3_WAVE - 1)) == 0) parts[threadIdx.x / CO3_WAVE][p] = part;
                }
                __syncthreads();
                if ((int)threadIdx.x < np) {
                    uint32_t mm = 0;
                    for (int w = 0; w < CV_BLOCK / CO3_WAVE; ++w) mm = mm > parts[w][threadIdx.x] ? mm : parts[w][threadIdx.x];
                    int cand = (int)(mm >> 23) - 127;
                    if (cand > 127) cand = 127;
                    if (seg_off[sg0 + threadIdx.x + 1] > seg_off[sg0 + threadIdx.x])       // an empty tensor keeps the clamp
                        atomicMax(anchor_u + sg0 + threadIdx.x, cand);
                }
                __syncthreads();
            }
            cur_seg = s_hi;
        }
    }
    absmax_flush(m, anchor_u + cur_seg, red);
}

// SCALED: the bias in its multiplier form (Sec. III (i) with the approximation of Sec. IV-B): the corrected
// gradient is multiplied by c before it is rounded onto the grid of the given anchor, and the level
// is divided by c again; one fp32 rounding per operation.
// NIB (alphabets of at most 16 symbols): the symbols leave two per byte, the earlier one in the low half, a
// user's row taking stride / 2 bytes.  A thread's elements start at a multiple of four, so the bytes it
// writes are its own.
template <bool HIST, bool SCALED, bool NIB = false>
__global__ __launch_bounds__(CV_BLOCK) void k_convert_ef(const float *__restrict__ g, float *__restrict__ err,
                                                          uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                          const int64_t *__restrict__ seg_off_g, int nseg,
                                                          const int32_t *__restrict__ anchor,
                                                          const float *__restrict__ scale, float gamma, co3_fmt fmt,
                                                          uint32_t *__restrict__ counts, int64_t per_block)
{
    const FmtC fc(fmt);
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    const int E = fc.E, M = fc.M, F = fc.F, K = fc.K, codemax = fc.codemax;
    // Users and ranges are taken in the reverse of the order in which the anchor pass read g, so that
    // the part of g that pass left in the last-level cache is read first.
    const int u = gridDim.y - 1 - blockIdx.y;
    const int64_t range = gridDim.x - 1 - blockIdx.x;
    const float *gu = g + (int64_t)u * stride;
    float *eu = err + (int64_t)u * stride;
    uint8_t *su = sym + (int64_t)u * (NIB ? stride / 2 : stride);
    const int32_t *anchor_u = anchor + (int64_t)u * nseg;
    const float *scale_u = SCALED ? scale + (int64_t)u * nseg : nullptr;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    // symbols of four consecutive elements from i (a multiple of four) on; one symbol of element j
    auto store_sym4 = [&](int64_t i, uint32_t q0, uint32_t q1, uint32_t q2, uint32_t q3) {
        if (NIB) *reinterpret_cast<uint16_t *>(su + (i >> 1)) = (uint16_t)(q0 | (q1 << 4) | (q2 << 8) | (q3 << 12));
        else *reinterpret_cast<uint32_t *>(su + i) = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
    };
    auto store_sym1 = [&](int64_t j, uint32_t q) {
        if (!NIB) su[j] = (uint8_t)q;
        else if ((j & 1) == 0) su[j >> 1] = (uint8_t)q;              // the even element writes the byte ...
        else su[j >> 1] = (uint8_t)(su[j >> 1] | (q << 4));          // ... the odd one, the same thread after it, joins
    };

    // per-wavefront private histogram: `copies` interleaved replicas of the K counters so that
    // lanes hitting one popular symbol spread over banks
    __shared__ uint32_t hist[CV_BLOCK / CO3_WAVE][HIST_SLOTS];
    const int copies = HIST_SLOTS / K > 32 ? 32 : HIST_SLOTS / K;
    uint32_t *myhist = hist[wave];
    const int mycopy = lane & (copies - 1);
    if (HIST) {
        for (int j = threadIdx.x; j < (CV_BLOCK / CO3_WAVE) * HIST_SLOTS; j += CV_BLOCK) (&hist[0][0])[j] = 0;
        __syncthreads();
    }

    int64_t beg = range * per_block;
    int64_t end = beg + per_block < n ? beg + per_block : n;

    // one element: correct, convert, new memory.  No contraction (build flag): one rounding per operation.
    auto convert1 = [&](float gv, float ev, int A, int e_min, float c, uint32_t &q) -> float {
        const float x = gv + gamma * ev;
        float v;
        co3_quantize(SCALED ? c * x : x, e_min, A, E, M, codemax, q, v);
        if (SCALED) v = v / c;
        return x - v;
    };
    // four elements of one thread, the symbols counted
    auto convert4 = [&](int64_t i, int A, float c, float4 gv, float4 ev) {
        const int e_min = A - F + 1;
        uint32_t q0, q1, q2, q3;
        float4 en;
        en.x = convert1(gv.x, ev.x, A, e_min, c, q0);
        en.y = convert1(gv.y, ev.y, A, e_min, c, q1);
        en.z = convert1(gv.z, ev.z, A, e_min, c, q2);
        en.w = convert1(gv.w, ev.w, A, e_min, c, q3);
        st_stream_f4(eu + i, en);
        store_sym4(i, q0, q1, q2, q3);
        if (HIST) {
            atomicAdd(&myhist[q0 * copies + mycopy], 1u);
            atomicAdd(&myhist[q1 * copies + mycopy], 1u);
            atomicAdd(&myhist[q2 * copies + mycopy], 1u);
            atomicAdd(&myhist[q3 * copies + mycopy], 1u);
        }
    };
    // elements [a0, a1) of one tensor, one per thread and step
    auto convert_part = [&](int64_t a0, int64_t a1, int64_t step, int sg) {
        const int A = anchor_u[sg];
        const float c = SCALED ? scale_u[sg] : 1.0f;
        for (int64_t j = a0; j < a1; j += step) {
            uint32_t q;
            eu[j] = convert1(gu[j], eu[j], A, A - F + 1, c, q);
            store_sym1(j, q);
            if (HIST) atomicAdd(&myhist[q * copies + mycopy], 1u);
        }
    };

    int64_t t0 = beg;
    while (t0 < end) {
        if (t0 + 2 * CV_TILE <= end) {       // two full tiles inside one tensor: all four loads first
            int s_a = co3_find_seg(seg_off, nseg, t0);
            int s_b = co3_find_seg(seg_off, nseg, t0 + 2 * CV_TILE - 1);
            if (s_a == s_b) {
                const int A = anchor_u[s_a];
                const float c = SCALED ? scale_u[s_a] : 1.0f;
                const int64_t i0 = t0 + (int64_t)threadIdx.x * CV_VEC, i1 = i0 + CV_TILE;
                float4 g0 = ld_stream_f4(gu + i0), e0 = ld_stream_f4(eu + i0);
                float4 g1 = ld_stream_f4(gu + i1), e1 = ld_stream_f4(eu + i1);
                convert4(i0, A, c, g0, e0);
                convert4(i1, A, c, g1, e1);
                t0 += 2 * CV_TILE;
                continue;
            }
        }
        int64_t t1 = t0 + CV_TILE < end ? t0 + CV_TILE : end;
        int s_lo = co3_find_seg(seg_off, nseg, t0);
        int s_hi = co3_find_seg(seg_off, nseg, t1 - 1);
        int64_t i = t0 + (int64_t)threadIdx.x * CV_VEC;
        if (s_lo == s_hi && i + CV_VEC <= t1) {
            convert4(i, anchor_u[s_lo], SCALED ? scale_u[s_lo] : 1.0f, ld_stream_f4(gu + i), ld_stream_f4(eu + i));
        } else if (s_lo == s_hi) {       // ragged tail inside one tensor
            convert_part(i, (i + CV_VEC < t1 ? i + CV_VEC : t1), 1, s_lo);
        } else if (i + CV_VEC <= t1) {
            // a tile that straddles tensors: the same loads and stores as a plain tile (a loop per tensor
            // part would put one memory latency per part into this block), each element under the anchor
            // of its own tensor
            const float4 gv = ld_stream_f4(gu + i), ev = ld_stream_f4(eu + i);
            const int sa = co3_find_seg(seg_off, nseg, i), sb = co3_find_seg(seg_off, nseg, i + CV_VEC - 1);
            if (sa == sb) {
                convert4(i, anchor_u[sa], SCALED ? scale_u[sa] : 1.0f, gv, ev);
            } else {
                const float ga[CV_VEC] = {gv.x, gv.y, gv.z, gv.w}, ea[CV_VEC] = {ev.x, ev.y, ev.z, ev.w};
                float en[CV_VEC];
                uint32_t q[CV_VEC];
#pragma unroll
                for (int k = 0; k < CV_VEC; ++k) {
                    const int sg = co3_find_seg(seg_off, nseg, i + k);
                    const int A = anchor_u[sg];
                    en[k] = convert1(ga[k], ea[k], A, A - F + 1, SCALED ? scale_u[sg] : 1.0f, q[k]);
                    if (HIST) atomicAdd(&myhist[q[k] * copies + mycopy], 1u);
                }
                st_stream_f4(eu + i, make_float4(en[0], en[1], en[2], en[3]));
                store_sym4(i, q[0], q[1], q[2], q[3]);
            }
        } else {                         // its ragged end, element by element
            for (int64_t j = i; j < t1; ++j) convert_part(j, j + 1, 1, co3_find_seg(seg_off, nseg, j));
        }
        t0 += CV_TILE;
    }

    if (HIST) {
        __syncthreads();
        for (int k = threadIdx.x; k < K; k += CV_BLOCK) {
            uint32_t c = 0;
            for (int w = 0; w < CV_BLOCK / CO3_WAVE; ++w)
                for (int r = 0; r < copies; ++r) c += hist[w][k * copies + r];
            if (c) atomicAdd(&counts[(int64_t)u * K + k], c);
        }
    }
}

// ------------------------------------------------------------------------------------------
// stand-alone histogram of symbol bytes (same LDS scheme), 16 symbols per thread per step
// ------------------------------------------------------------------------------------------
#define HS_VEC 16
#define HS_TILE (CV_BLOCK * HS_VEC)

__global__ __launch_bounds__(CV_BLOCK) void k_histogram(const uint8_t *__restrict__ sym, int64_t n, int64_t stride,
                                                         int K, uint32_t *__restrict__ counts, int64_t per_block)
{
    const int u = blockIdx.y;
    const uint8_t *su = sym + (int64_t)u * stride;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    __shared__ uint32_t hist[CV_BLOCK / CO3_WAVE][HIST_SLOTS];
    const int copies = HIST_SLOTS / K > 32 ? 32 : HIST_SLOTS / K;
    uint32_t *myhist = hist[wave];
    const int mycopy = lane & (copies - 1);
    for (int j = threadIdx.x; j < (CV_BLOCK / CO3_WAVE) * HIST_SLOTS; j += CV_BLOCK) (&hist[0][0])[j] = 0;
    __syncthreads();

    int64_t beg = (int64_t)blockIdx.x * per_block;
    int64_t end = beg + per_block < n ? beg + per_block : n;
    for (int64_t t0 = beg; t0 < end; t0 += HS_TILE) {
        int64_t i = t0 + (int64_t)threadIdx.x * HS_VEC;
        if (i + HS_VEC <= end) {
            uint4 v = *reinterpret_cast<const uint4 *>(su + i);
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    uint32_t q = (w[a] >> (8 * b)) & 0xffu;
                    if (q < (uint32_t)K) atomicAdd(&myhist[q * copies + mycopy], 1u);
                }
        } else {
            for (int64_t j = i; j < end; ++j) {
                uint32_t q = su[j];
                if (q < (uint32_t)K) atomicAdd(&myhist[q * copies + mycopy], 1u);
            }
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += CV_BLOCK) {
        uint32_t c = 0;
        for (int w = 0; w < CV_BLOCK / CO3_WAVE; ++w)
            for (int r = 0; r < copies; ++r) c += hist[w][k * copies + r];
        if (c) atomicAdd(&counts[(int64_t)u * K + k], c);
    }
}

// ------------------------------------------------------------------------------------------
// symbol counts per (user, tensor) -- the statistics behind one code per layer (Sec. III (ii)):
// the same LDS scheme, emptied into counts[u][tensor] whenever the block moves to another tensor
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(CV_BLOCK) void k_histogram_layers(const uint8_t *__restrict__ sym, int64_t n,
                                                                int64_t stride, int K,
                                                                const int64_t *__restrict__ seg_off_g, int nseg,
                                                                int pool_users, uint32_t *__restrict__ counts,
                                                                int64_t per_block)
{
    const int u = blockIdx.y;
    const int row = pool_users ? 0 : u;       // pooled: all users add into one [nseg][K] table
    const uint8_t *su = sym + (int64_t)u * stride;
    const int lane = threadIdx.x & (CO3_WAVE - 1);
    const int wave = threadIdx.x / CO3_WAVE;
    __shared__ uint32_t hist[CV_BLOCK / CO3_WAVE][HIST_SLOTS];
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    const int copies = HIST_SLOTS / K > 32 ? 32 : HIST_SLOTS / K;
    uint32_t *myhist = hist[wave];
    const int mycopy = lane & (copies - 1);
    for (int j = threadIdx.x; j < (CV_BLOCK / CO3_WAVE) * HIST_SLOTS; j += CV_BLOCK) (&hist[0][0])[j] = 0;
    __syncthreads();

    // adds the block's counters to tensor sg of this user and clears them (block-uniform call)
    auto flush = [&](int sg) {
        __syncthreads();
        uint32_t *dst = counts + ((int64_t)row * nseg + sg) * K;
        for (int k = threadIdx.x; k < K; k += CV_BLOCK) {
            uint32_t c = 0;
            for (int w = 0; w < CV_BLOCK / CO3_WAVE; ++w)
                for (int r = 0; r < copies; ++r) {
                    c += hist[w][k * copies + r];
                    hist[w][k * copies + r] = 0;
                }
            if (c) atomicAdd(&dst[k], c);
        }
        __syncthreads();
    };
    auto count1 = [&](uint32_t q) {
        if (q < (uint32_t)K) atomicAdd(&myhist[q * copies + mycopy], 1u);
    };

    int64_t beg = (int64_t)blockIdx.x * per_block;
    int64_t end = beg + per_block < n ? beg + per_block : n;
    if (beg >= end) return;
    int cur_seg = co3_find_seg(seg_off, nseg, beg);
    for (int64_t t0 = beg; t0 < end; t0 += HS_TILE) {
        const int64_t t1 = t0 + HS_TILE < end ? t0 + HS_TILE : end;
        const int s_lo = co3_find_seg(seg_off, nseg, t0), s_hi = co3_find_seg(seg_off, nseg, t1 - 1);
        if (s_lo == s_hi) {
            if (s_lo != cur_seg) {
                flush(cur_seg);
                cur_seg = s_lo;
            }
            const int64_t i = t0 + (int64_t)threadIdx.x * HS_VEC;
            if (i + HS_VEC <= t1) {
                uint4 v = *reinterpret_cast<const uint4 *>(su + i);
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) count1((w[a] >> (8 * b)) & 0xffu);
            } else {
                for (int64_t j = i; j < t1; ++j) count1(su[j]);
            }
        } else {
            flush(cur_seg);
            for (int sg = s_lo; sg <= s_hi; ++sg) {
                const int64_t a0 = seg_off[sg] > t0 ? seg_off[sg] : t0;
                const int64_t a1 = seg_off[sg + 1] < t1 ? seg_off[sg + 1] : t1;
                for (int64_t j = a0 + threadIdx.x; j < a1; j += CV_BLOCK) count1(su[j]);
                flush(sg);
            }
            cur_seg = s_hi;
        }
    }
    flush(cur_seg);
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
static int64_t per_block_for(int64_t n, int U, int64_t tile, int *blocks_out, int K = 0, bool few = false)
{
    // about 8 blocks per compute unit in total, each a whole number of tiles; half as many when every
    // block ends by adding up to 256 counters into the same few cache lines; (few) at least two tiles per
    // block where every block ends with an atomic on one word per tensor
    int64_t target_blocks = (K >= 128 ? 1024 : 2048) / (U > 0 ? U : 1);
    int64_t tiles = (n + tile - 1) / tile;
    if (few && target_blocks > tiles / 2) target_blocks = tiles / 2;
    if (target_blocks < 1) target_blocks = 1;
    int64_t tiles_per_block = (tiles + target_blocks - 1) / target_blocks;
    if (tiles_per_block < 1) tiles_per_block = 1;
    int64_t blocks = (tiles + tiles_per_block - 1) / tiles_per_block;
    if (blocks < 1) blocks = 1;
    *blocks_out = (int)blocks;
    return tiles_per_block * tile;
}

hipError_t co3_launch_fill(int32_t *a, int64_t na, int32_t va, uint32_t *b, int64_t nb, hipStream_t st, uint32_t vb)
{
    int64_t m = na > nb ? na : nb;
    if (m <= 0) return hipSuccess;
    int blocks = (int)((m + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    Co3LaunchTimer tm(CO3_K_FILL, st);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks), dim3(256), 0, st, a, na, va, b, nb, vb);
    return hipGetLastError();
}

hipError_t co3_launch_absmax(const float *g, int64_t n, int U, int64_t stride, const int64_t *seg_off, int nseg,
                             int32_t *anchor, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int blocks;
    int64_t pb = per_block_for(n, U, AM_TILE, &blocks, 0, true);
    Co3LaunchTimer tm(CO3_K_ABSMAX, st);
    hipLaunchKernelGGL(k_absmax, dim3(blocks, U), dim3(CV_BLOCK), 0, st, g, n, stride, seg_off, nseg, anchor, pb);
    return hipGetLastError();
}

hipError_t co3_launch_convert(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride,
                              const int64_t *seg_off, int nseg, const int32_t *anchor, const float *scale, float gamma,
                              co3_fmt fmt, uint32_t *counts, hipStream_t st, int sym_nib)
{
    if (n <= 0) return hipSuccess;
    if (sym_nib && (!counts || scale || (1 << (1 + fmt.exp_bits + fmt.mant_bits)) > 16)) return hipErrorInvalidValue;
    int blocks;
    int64_t pb = per_block_for(n, U, CV_TILE, &blocks, counts ? 1 << (1 + fmt.exp_bits + fmt.mant_bits) : 0);
    Co3LaunchTimer tm(CO3_K_CONVERT, st);
    const dim3 grid(blocks, U), block(CV_BLOCK);
    if (sym_nib) {
        hipLaunchKernelGGL((k_convert_ef<true, false, true>), grid, block, 0, st, g, err, sym, n, stride, seg_off, nseg, anchor,
                           scale, gamma, fmt, counts, pb);
        return hipGetLastError();
    }
#define CO3_CONVERT_LAUNCH(H, S)                                                                                     \
    hipLaunchKernelGGL((k_convert_ef<H, S>), grid, block, 0, st, g, err, sym, n, stride, seg_off, nseg, anchor, scale, \
                       gamma, fmt, counts, pb)
    if (counts && scale) CO3_CONVERT_LAUNCH(true, true);
    else if (counts) CO3_CONVERT_LAUNCH(true, false);
    else if (scale) CO3_CONVERT_LAUNCH(false, true);
    else CO3_CONVERT_LAUNCH(false, false);
#undef CO3_CONVERT_LAUNCH
    return hipGetLastError();
}

hipError_t co3_launch_histogram(const uint8_t *sym, int64_t n, int U, int64_t stride, int K, uint32_t *counts,
                                hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int blocks;
    int64_t pb = per_block_for(n, U, HS_TILE, &blocks, K);
    Co3LaunchTimer tm(CO3_K_HISTOGRAM, st);
    hipLaunchKernelGGL(k_histogram, dim3(blocks, U), dim3(CV_BLOCK), 0, st, sym, n, stride, K, counts, pb);
    return hipGetLastError();
}

hipError_t co3_launch_histogram_layers(const uint8_t *sym, int64_t n, int U, int64_t stride, int K,
                                       const int64_t *seg_off, int nseg, int pool_users, uint32_t *counts,
                                       hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int blocks;
    int64_t pb = per_block_for(n, U, HS_TILE, &blocks, K);
    Co3LaunchTimer tm(CO3_K_HISTOGRAM, st);
    hipLaunchKernelGGL(k_histogram_layers, dim3(blocks, U), dim3(CV_BLOCK), 0, st, sym, n, stride, K, seg_off, nseg,
                       pool_users, counts, pb);
    return hipGetLastError();
}
