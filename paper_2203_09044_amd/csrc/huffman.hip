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

hipError_t co3_launch_build_code(const uint32_t *weights, int U, int K, void *codes, int32_t *status, hipStream_t st,
                                 int nrep, uint32_t *sums_out)
{
    if (U <= 0) return hipSuccess;
    Co3LaunchTimer tm(CO3_K_BUILD, st);
    hipLaunchKernelGGL(k_build_code, dim3(U), dim3(HB_BLOCK), 0, st, weights, K, reinterpret_cast<char *>(codes),
                       status, nrep, sums_out);
    return hipGetLastError();
}
