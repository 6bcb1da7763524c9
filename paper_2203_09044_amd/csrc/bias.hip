// The bias rule of the paper in its multiplier form (Sec. III (i), Eq. (exp bias); Sec. IV-B, "fp exponent
// bias", Eq. (approximate)): statistics of the corrected gradient per (user, tensor), a GenNorm fit
// by moment matching, and the printed fourth-degree polynomial in the fitted shape divided by the
// fitted scale.
#include "co3_dev.h"
#include "kernels.h"

#define MO_BLOCK 256
#define MO_VEC 4
#define MO_UNROLL 4
#define MO_TILE (MO_BLOCK * MO_VEC * MO_UNROLL)   // elements per block step: 4 x (16 B g + 16 B m) in flight per thread

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int d = CO3_WAVE / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d, CO3_WAVE);
    return v;
}

// Block-wide sums, then two fp64 atomics per block and tensor.  Called under block-uniform conditions.
__device__ __forceinline__ void moments_flush(double s1, double s2, double *sums_us, double (*red)[2])
{
    s1 = wave_sum_f64(s1);
    s2 = wave_sum_f64(s2);
    if ((threadIdx.x & (CO3_WAVE - 1)) == 0) {
        red[threadIdx.x / CO3_WAVE][0] = s1;
        red[threadIdx.x / CO3_WAVE][1] = s2;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < MO_BLOCK / CO3_WAVE; ++w) {
            a += red[w][0];
            b += red[w][1];
        }
        if (b != 0.0) {
            atomicAdd(sums_us, a);
            atomicAdd(sums_us + 1, b);
        }
    }
    __syncthreads();
}

// sums[u][tensor] = (sum |x|, sum x^2) of x = fl32(g + fl32(gamma * m)), accumulated in fp64
__global__ __launch_bounds__(MO_BLOCK) void k_moments(const float *__restrict__ g, const float *__restrict__ err,
                                                       int64_t n, int64_t stride,
                                                       const int64_t *__restrict__ seg_off_g, int nseg, float gamma,
                                                       double *__restrict__ sums, int64_t per_block)
{
    const int u = blockIdx.y;
    const float *gu = g + (int64_t)u * stride;
    const float *eu = err + (int64_t)u * stride;
    double *sums_u = sums + (int64_t)u * nseg * 2;
    __shared__ double red[MO_BLOCK / CO3_WAVE][2];
    __shared__ int64_t seg_cache[CO3_SEG_CACHE];
    const int64_t *seg_off = co3_cache_segs(seg_off_g, nseg, seg_cache);
    int64_t beg = (int64_t)blockIdx.x * per_block;
    int64_t end = beg + per_block < n ? beg + per_block : n;
    if (beg >= end) return;

    double s1 = 0.0, s2 = 0.0;
    auto add1 = [&](float gv, float ev) {
        const float x = gv + gamma * ev;      // no contraction (build flag): as the conversion computes it
        const double xd = (double)x;
        s1 += fabs(xd);
        s2 += xd * xd;
    };
    int cur_seg = co3_find_seg(seg_off, nseg, beg);
    for (int64_t t0 = beg; t0 < end; t0 += MO_TILE) {
        int64_t t1 = t0 + MO_TILE < end ? t0 + MO_TILE : end;
        int s_lo = co3_find_seg(seg_off, nseg, t0);
        int s_hi = co3_find_seg(seg_off, nseg, t1 - 1);
        int64_t i = t0 + (int64_t)threadIdx.x * MO_VEC;
        if (s_lo == s_hi) {
            if (s_lo != cur_seg) {       // block-uniform branch
                moments_flush(s1, s2, sums_u + 2 * cur_seg, red);
                s1 = s2 = 0.0;
                cur_seg = s_lo;
            }
            if (t1 - t0 == MO_TILE) {
                float4 gv[MO_UNROLL], ev[MO_UNROLL];
#pragma unroll
                for (int k = 0; k < MO_UNROLL; ++k) {
                    gv[k] = *reinterpret_cast<const float4 *>(gu + i + (int64_t)k * (MO_BLOCK * MO_VEC));
                    ev[k] = *reinterpret_cast<const float4 *>(eu + i + (int64_t)k * (MO_BLOCK * MO_VEC));
                }
#pragma unroll
                for (int k = 0; k < MO_UNROLL; ++k) {
                    add1(gv[k].x, ev[k].x);
                    add1(gv[k].y, ev[k].y);
                    add1(gv[k].z, ev[k].z);
                    add1(gv[k].w, ev[k].w);
                }
            } else {
                for (int64_t j = t0 + threadIdx.x; j < t1; j += MO_BLOCK) add1(gu[j], eu[j]);
            }
        } else {
            // The tile straddles tensors.  Its elements are loaded once, all loads in flight together as in
            // the plain case (a loop per tensor part would put one memory latency per part into this block,
            // and the kernel ends with its slowest block); then every part is summed from registers.
            moments_flush(s1, s2, sums_u + 2 * cur_seg, red);
            float x[MO_UNROLL][MO_VEC];
#pragma unroll
            for (int k = 0; k < MO_UNROLL; ++k) {
                const int64_t j0 = i + (int64_t)k * (MO_BLOCK * MO_VEC);
                float gq[MO_VEC], eq[MO_VEC];
                if (j0 + MO_VEC <= t1) {
                    const float4 gv = *reinterpret_cast<const float4 *>(gu + j0), ev = *reinterpret_cast<const float4 *>(eu + j0);
                    gq[0] = gv.x; gq[1] = gv.y; gq[2] = gv.z; gq[3] = gv.w;
                    eq[0] = ev.x; eq[1] = ev.y; eq[2] = ev.z; eq[3] = ev.w;
                } else {
#pragma unroll
                    for (int c = 0; c < MO_VEC; ++c) {
                        gq[c] = j0 + c < t1 ? gu[j0 + c] : 0.0f;
                        eq[c] = j0 + c < t1 ? eu[j0 + c] : 0.0f;
                    }
                }
#pragma unroll
                for (int c = 0; c < MO_VEC; ++c) x[k][c] = gq[c] + gamma * eq[c];   // as the conversion computes it
            }
            for (int sg = s_lo; sg <= s_hi; ++sg) {
                const int64_t a0 = seg_off[sg], a1 = seg_off[sg + 1];
                s1 = s2 = 0.0;
#pragma unroll
                for (int k = 0; k < MO_UNROLL; ++k)
#pragma unroll
                    for (int c = 0; c < MO_VEC; ++c) {
                        const int64_t j = i + (int64_t)k * (MO_BLOCK * MO_VEC) + c;
                        const double xd = j >= a0 && j < a1 && j < t1 ? (double)x[k][c] : 0.0;
                        s1 += fabs(xd);
                        s2 += xd * xd;
                    }
                moments_flush(s1, s2, sums_u + 2 * sg, red);
            }
            s1 = s2 = 0.0;
            cur_seg = s_hi;
        }
    }
    moments_flush(s1, s2, sums_u + 2 * cur_seg, red);
}

// (E|X|)^2 / E[X^2] of GenNorm(beta) = Gamma(2/b)^2 / (Gamma(1/b) Gamma(3/b)): increasing, 0 .. 3/4
__device__ __forceinline__ double gennorm_ratio(double beta)
{
    return exp(2.0 * lgamma(2.0 / beta) - lgamma(1.0 / beta) - lgamma(3.0 / beta));
}

#define FIT_BETA_LO 0.05
#define FIT_BETA_HI 50.0
#define FIT_ROUNDS 8      // each round narrows the bracket's log-width 65-fold: log(1000) / 65^8 = 2e-14

// One wavefront per (user, tensor).  The shape beta solves ratio(beta) = s1^2 / (count * s2); the 64 lanes
// evaluate the ratio at 64 geometrically spaced points of the bracket per round.  The scale alpha
// reproduces the second moment; the multiplier is the printed polynomial in beta (beta limited to the
// plotted range 0.4 .. 1.6) over alpha, kept within [2^-96, 2^96]; a tensor of zeros gets multiplier 1.
__global__ __launch_bounds__(CO3_WAVE) void k_bias_scale(const double *__restrict__ sums,
                                                          const int64_t *__restrict__ seg_off, int nseg, int64_t n,
                                                          float *__restrict__ scale, double *__restrict__ fit)
{
    const int sg = blockIdx.x, u = blockIdx.y;
    const int lane = threadIdx.x;
    const int64_t idx = (int64_t)u * nseg + sg;
    const double s1 = sums[2 * idx], s2 = sums[2 * idx + 1];
    const int64_t count = seg_off ? seg_off[sg + 1] - seg_off[sg] : n;
    double beta = 1.0, alpha = 0.0;
    if (count > 0 && s2 > 0.0) {
        const double rho = s1 * s1 / ((double)count * s2);
        double lo = FIT_BETA_LO, hi = FIT_BETA_HI;
        if (rho <= gennorm_ratio(lo)) {
            hi = lo;
        } else if (rho >= gennorm_ratio(hi)) {
            lo = hi;
        } else {
            for (int round = 0; round < FIT_ROUNDS; ++round) {
                const double step = log(hi / lo) / 65.0;
                const double mine = lo * exp(step * (double)(lane + 1));
                const bool below = gennorm_ratio(mine) < rho;
                // the ratio is increasing: lanes below the target form a prefix
                const int nb = __popcll(__ballot(below));
                const double new_lo = nb == 0 ? lo : __shfl(mine, nb - 1, CO3_WAVE);
                const double new_hi = nb == CO3_WAVE ? hi : __shfl(mine, nb, CO3_WAVE);
                lo = new_lo;
                hi = new_hi;
            }
        }
        beta = 0.5 * (lo + hi);
        alpha = sqrt(s2 / (double)count * exp(lgamma(1.0 / beta) - lgamma(3.0 / beta)));
    }
    if (lane == 0) {
        float c = 1.0f;
        if (alpha > 0.0) {
            const double b = beta < 0.4 ? 0.4 : (beta > 1.6 ? 1.6 : beta);
            double v = (0.46 - 2.85 * b + 5.37 * b * b - 2.85 * b * b * b + 0.52 * b * b * b * b) / alpha;
            const double lim = 7.9228162514264338e28;      // 2^96
            if (!(v < lim)) v = lim;
            if (!(v > 1.0 / lim)) v = 1.0 / lim;
            c = (float)v;
        }
        scale[idx] = c;
        if (fit) {
            fit[2 * idx] = beta;
            fit[2 * idx + 1] = alpha;
        }
    }
}

hipError_t co3_launch_moments(const float *g, const float *err, int64_t n, int U, int64_t stride,
                              const int64_t *seg_off, int nseg, float gamma, double *sums, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    int64_t target_blocks = 2048 / U;
    const int64_t tiles = (n + MO_TILE - 1) / MO_TILE;
    if (target_blocks > tiles / 4) target_blocks = tiles / 4;   // every block ends with two atomics per tensor: few blocks end at once
    if (target_blocks < 1) target_blocks = 1;
    int64_t tiles_per_block = (tiles + target_blocks - 1) / target_blocks;
    if (tiles_per_block < 1) tiles_per_block = 1;
    const int64_t blocks = (tiles + tiles_per_block - 1) / tiles_per_block;
    Co3LaunchTimer tm(CO3_K_MOMENTS, st);
    hipLaunchKernelGGL(k_moments, dim3((unsigned)blocks, U), dim3(MO_BLOCK), 0, st, g, err, n, stride, seg_off, nseg,
                       gamma, sums, tiles_per_block * MO_TILE);
    return hipGetLastError();
}

hipError_t co3_launch_bias_scale(const double *sums, int64_t n, int U, const int64_t *seg_off, int nseg, float *scale,
                                 double *fit, hipStream_t st)
{
    Co3LaunchTimer tm(CO3_K_BIAS_SCALE, st);
    hipLaunchKernelGGL(k_bias_scale, dim3(nseg, U), dim3(CO3_WAVE), 0, st, sums, seg_off, nseg, n, scale, fit);
    return hipGetLastError();
}
