// Huffman code construction (Sec. III (ii)): one workgroup per user builds code lengths,
// canonical codewords and the decoder tables from K <= 256 integer weights.
#include "co3_dev.h"
#include "co3_huffman.h"
#include "kernels.h"

#define HB_BLOCK 256

// nrep > 1: the weights of a user arrive as nrep partial tables [nrep][U][K] (partial counts of groups of
// workgroups); they are added up here and the sums also go to sums_out [U][K].
__global__ __launch_bounds__(HB_BLOCK) void k_build_code(const uint32_t *__restrict__ weights, int K, char *codes,
                                                          int32_t *status, int nrep, uint32_t *__restrict__ sums_out)
{
    const int u = blockIdx.x;
    const int tid = threadIdx.x;
    Co3Code *out = reinterpret_cast<Co3Code *>(codes + (size_t)u * CO3_CODE_BYTES);
    __shared__ Co3BuildLds lds;
    uint32_t wt[1] = {0u};
    if (tid < K) {
        const size_t rep_stride = (size_t)gridDim.x * K;
        const uint32_t *w0 = weights + (size_t)u * K + tid;
        int r = 0;
        for (; r + 8 <= nrep; r += 8) {          // the loads of a batch are independent
            uint32_t part[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) part[k] = w0[(r + k) * rep_stride];
#pragma unroll
            for (int k = 0; k < 8; ++k) wt[0] += part[k];
        }
        for (; r < nrep; ++r) wt[0] += w0[r * rep_stride];
        if (sums_out) sums_out[(size_t)u * K + tid] = wt[0];
    }
    co3_build_code_group<HB_BLOCK>(lds, tid, wt, K, out, nullptr, status, Co3BlockSync());
}

// What is left of a user's steps before compression when a resident grid has converted everything but the
// ragged end of the vector (Algorithm 1, the user's conversion, memory update and code design; Sec. III
// (i)-(iii)): one workgroup per user converts elements [n_full, n) with the user's anchor, counts their
// symbols, adds the grid's partial count tables to them and builds the user's code.
__global__ __launch_bounds__(HB_BLOCK) void k_user_finish(const float *__restrict__ g, float *__restrict__ err,
                                                           uint8_t *__restrict__ sym, int64_t n, int64_t n_full,
                                                           int64_t stride, const int64_t *__restrict__ seg_off, int nseg,
                                                           const int32_t *__restrict__ anchor, float gamma,
                                                           co3_fmt fmt, int sym_nib, const uint32_t *__restrict__ counts_rep,
                                                           int nrep, uint32_t *__restrict__ counts, char *codes,
                                                           int32_t *status, int first_user, int U)
{
    const FmtC fc(fmt);
    const int K = fc.K;
    const int tid = threadIdx.x;
    const int u = first_user + blockIdx.x;       // users first_user .. first_user + gridDim.x - 1 of the batch of U
    __shared__ Co3BuildLds lds;
    __shared__ uint32_t hist[256];
    hist[tid] = 0u;
    // the partial tables are requested before the ragged end is converted
    uint32_t part_sum = 0;
    if (tid < K) {
        for (int r0 = 0; r0 < nrep; r0 += 8) {          // the loads of a batch are independent
            uint32_t part[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) part[k] = r0 + k < nrep ? counts_rep[((size_t)(r0 + k) * U + u) * K + tid] : 0u;
#pragma unroll
            for (int k = 0; k < 8; ++k) part_sum += part[k];
        }
    }
    __syncthreads();
    // one anchor per (user, tensor): anchor is [U][nseg]
    const float *gu = g + (int64_t)u * stride;
    float *eu = err + (int64_t)u * stride;
    uint8_t *su = sym + (int64_t)u * (sym_nib ? stride / 2 : stride);
    // four consecutive elements per thread and step (n_full is a multiple of four: with two symbols per byte
    // the bytes a thread writes are its own)
    for (int64_t i = n_full + 4 * (int64_t)tid; i < n; i += 4 * HB_BLOCK) {
        uint32_t q[4] = {0u, 0u, 0u, 0u};
        const int cnt = n - i < 4 ? (int)(n - i) : 4;
        for (int c = 0; c < cnt; ++c) {
            const float x = gu[i + c] + gamma * eu[i + c];          // no contraction (build flag): one rounding per operation
            const int A = anchor[(int64_t)u * nseg + co3_find_seg(seg_off, nseg, i + c)];
            float v;
            co3_quantize(x, A - fc.F + 1, A, fc.E, fc.M, fc.codemax, q[c], v);
            eu[i + c] = x - v;
            atomicAdd(&hist[q[c]], 1u);
        }
        if (sym_nib) {
            su[i >> 1] = (uint8_t)(q[0] | (q[1] << 4));
            if (cnt > 2) su[(i >> 1) + 1] = (uint8_t)(q[2] | (q[3] << 4));
        } else {
            for (int c = 0; c < cnt; ++c) su[i + c] = (uint8_t)q[c];
        }
    }
    __syncthreads();
    uint32_t wt[1] = {0u};
    if (tid < K) {
        wt[0] = hist[tid] + part_sum;
        counts[(size_t)u * K + tid] = wt[0];
    }
    co3_build_code_group<HB_BLOCK>(lds, tid, wt, K, reinterpret_cast<Co3Code *>(codes + (size_t)u * CO3_CODE_BYTES), nullptr,
                                   status, Co3BlockSync());
}

hipError_t co3_launch_user_finish(const float *g, float *err, uint8_t *sym, int64_t n, int64_t n_full, int64_t stride, int U,
                                  const int64_t *seg_off, int nseg, const int32_t *anchor, float gamma, co3_fmt fmt,
                                  int sym_nib, const uint32_t *counts_rep, int nrep, uint32_t *counts, void *codes,
                                  int32_t *status, hipStream_t st, int first_user, int users)
{
    if (U <= 0 || users <= 0) return hipSuccess;
    Co3LaunchTimer tm(CO3_K_BUILD, st);
    hipLaunchKernelGGL(k_user_finish, dim3(users), dim3(HB_BLOCK), 0, st, g, err, sym, n, n_full, stride, seg_off, nseg, anchor, gamma, fmt,
                       sym_nib, counts_rep, nrep, counts, reinterpret_cast<char *>(codes), status, first_user, U);
    return hipGetLastError();
}

hipError_t co3_launch_build_code(const uint32_t *weights, int U, int K, void *codes, int32_t *status, hipStream_t st,
                                 int nrep, uint32_t *sums_out)
{
    if (U <= 0) return hipSuccess;
    Co3LaunchTimer tm(CO3_K_BUILD, st);
    hipLaunchKernelGGL(k_build_code, dim3(U), dim3(HB_BLOCK), 0, st, weights, K, reinterpret_cast<char *>(codes),
                       status, nrep, sums_out);
    return hipGetLastError();
}
