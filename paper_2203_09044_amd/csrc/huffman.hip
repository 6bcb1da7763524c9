// Huffman code construction (Sec. III (ii)): one workgroup per user builds code lengths,
// canonical codewords and the decoder tables from K <= 256 integer weights.
#include "co3_dev.h"
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

    __shared__ uint64_t key[HB_BLOCK];        // (weight << 8 | symbol), inactive symbols sort last
    __shared__ uint64_t node_w[2 * HB_BLOCK]; // weights of merged nodes (index >= nact)
    __shared__ uint16_t parent[2 * HB_BLOCK];
    __shared__ __attribute__((aligned(4))) uint8_t len_s[HB_BLOCK];   // also read as words
    __shared__ uint32_t cnt_s[66];
    __shared__ uint64_t first_s[66];
    __shared__ uint32_t base_s[66];
    __shared__ uint8_t sorted_s[HB_BLOCK];
    __shared__ uint32_t maxlen_s;

    uint32_t wt = 0u;
    if (tid < K) {
        const size_t rep_stride = (size_t)gridDim.x * K;
        for (int r = 0; r < nrep; ++r) wt += weights[r * rep_stride + (size_t)u * K + tid];
        if (sums_out) sums_out[(size_t)u * K + tid] = wt;
    }
    const uint64_t mykey = wt ? (((uint64_t)wt << 8) | (uint64_t)tid) : ~0ull;
    key[tid] = mykey;
    len_s[tid] = 0;
    sorted_s[tid] = 0;
    if (tid < 66) {
        cnt_s[tid] = 0;
        first_s[tid] = 0;
        base_s[tid] = 0;
    }
    if (tid == 0) maxlen_s = 0;
    const int nact = __syncthreads_count(wt != 0u);

    // leaves in (weight, symbol) order: every thread counts the keys below its own (all threads read the
    // same entry at the same time, a broadcast) and stores its key at that position; the symbols without
    // a weight share one key and are ordered among themselves by their index
    {
        int below = 0;
        for (int j = 0; j < K; ++j) {        // entries from K on hold the no-weight key and stay where they are
            const uint64_t kj = key[j];
            below += (kj < mykey || (kj == mykey && j < tid)) ? 1 : 0;
        }
        if (tid >= K) below = tid;
        __syncthreads();
        key[below] = mykey;
        __syncthreads();
    }

    // two-queue merge: nodes 0..nact-1 are the sorted leaves, nact..2*nact-2 the merged nodes in
    // creation order; a leaf wins a weight tie against a merged node
    // One lane runs the merge.  A step reads the two front entries of each queue and takes one of three
    // outcomes: two leaves (the second leaf is not above the first node), two nodes (the second node is
    // below the first leaf), or the first leaf with the first node (their order does not matter to the
    // sum or to the parent links).  Both queues are padded with an unreachable weight, so no bounds
    // test is needed; the node created by a step is written before the next step reads the fronts.
    const uint64_t INF = ~0ull;     // weights stay below 2^40, so INF never wins while a queue has entries
    __shared__ uint64_t leaf_q[HB_BLOCK + 4];
    leaf_q[tid] = tid < nact ? (key[tid] >> 8) : INF;
    if (tid < 4) leaf_q[HB_BLOCK + tid] = INF;
    node_w[tid] = INF;
    node_w[HB_BLOCK + tid] = INF;
    __syncthreads();
    if (tid == 0 && nact >= 2) {
        int q1 = 0, q2 = nact;
        for (int next = nact; next < 2 * nact - 1; ++next) {
            const uint64_t L0 = leaf_q[q1], L1 = leaf_q[q1 + 1];
            const uint64_t N0 = node_w[q2], N1 = node_w[q2 + 1];
            uint64_t wsum;
            if (L1 <= N0) {
                wsum = L0 + L1;
                parent[q1] = (uint16_t)next;
                parent[q1 + 1] = (uint16_t)next;
                q1 += 2;
            } else if (N1 < L0) {
                wsum = N0 + N1;
                parent[q2] = (uint16_t)next;
                parent[q2 + 1] = (uint16_t)next;
                q2 += 2;
            } else {
                wsum = L0 + N0;
                parent[q1] = (uint16_t)next;
                parent[q2] = (uint16_t)next;
                ++q1;
                ++q2;
            }
            node_w[next] = wsum;
        }
    }
    __syncthreads();

    // code length = depth of the leaf
    if (tid < nact) {
        int depth;
        if (nact == 1) {
            depth = 1;
        } else {
            const int root = 2 * nact - 2;
            depth = 0;
            for (int v = tid; v != root && depth < 255; v = parent[v]) ++depth;
        }
        int s = (int)(key[tid] & 0xffu);
        int dl = depth > 64 ? 64 : depth;
        len_s[s] = (uint8_t)dl;
        atomicAdd(&cnt_s[dl], 1u);
        atomicMax(&maxlen_s, (uint32_t)depth);
    }
    __syncthreads();
    const uint32_t maxlen = maxlen_s;
    if (tid == 0 && maxlen > CO3_MAX_CODE_LEN) co3_raise(status, CO3_EINVAL);

    // canonical numbering: first code of length l is sum_{j<l} count[j] << (l - j)
    if (tid >= 1 && tid <= 64) {
        uint64_t first = 0;
        uint32_t base = 0;
        for (int j = 1; j < tid; ++j) {
            first += (uint64_t)cnt_s[j] << (tid - j);
            base += cnt_s[j];
        }
        first_s[tid] = first;
        base_s[tid] = base;
    }
    __syncthreads();

    {
        uint32_t l = len_s[tid];
        uint64_t enc = 0;
        if (l) {
            // symbols below this one with the same length, four length bytes per LDS word
            uint32_t rank = 0;
            const uint32_t *len_w = reinterpret_cast<const uint32_t *>(len_s);
            const uint32_t pat = l * 0x01010101u;
            for (int j = 0; j <= tid >> 2; ++j) {
                uint32_t x = len_w[j] ^ pat;                       // zero bytes where the length matches
                if (j == tid >> 2) x |= ~0u << (8 * (tid & 3));    // only the symbols below this one
                const uint32_t z = ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);   // 0x80 per zero byte
                rank += (uint32_t)__builtin_popcount(z);
            }
            uint64_t code = first_s[l] + rank;
            sorted_s[base_s[l] + rank] = (uint8_t)tid;
            enc = (code << 6) | (uint64_t)(l & 63u);
        }
        out->len[tid] = (uint8_t)l;
        out->enc[tid] = enc;
    }
    __syncthreads();

    if (tid < 65) out->first_code[tid] = first_s[tid];
    if (tid < 66) {
        out->count[tid] = (uint16_t)cnt_s[tid];
        out->base[tid] = (uint16_t)base_s[tid];
    }
    out->sorted[tid] = sorted_s[tid];
    uint32_t lut_bits = maxlen < 1 ? 1 : (maxlen > CO3_LUT_BITS_MAX ? CO3_LUT_BITS_MAX : maxlen);
    if (tid == 0) {
        out->nact = (uint32_t)nact;
        out->maxlen = maxlen;
        out->lut_bits = lut_bits;
        out->reserved = 0;
    }

    // decoder table: entry i decodes the lut_bits-bit prefix i by the canonical rule.  Canonical
    // codewords grow with their length, so the prefixes resolved by length <= l form the range
    // [0, limit[l]) with limit[l] = (first_code[l] + count[l]) << (lut_bits - l): the entry's length is
    // the first l whose limit exceeds i.
    __shared__ uint32_t limit_s[CO3_LUT_BITS_MAX + 2];
    if (tid >= 1 && tid <= (int)lut_bits) {
        uint64_t lim = (first_s[tid] + cnt_s[tid]) << (lut_bits - tid);
        limit_s[tid] = lim > (1ull << lut_bits) ? (1u << lut_bits) : (uint32_t)lim;
    }
    __syncthreads();
    // (the limits do not decrease with the length: counting the limits at or below i gives the length;
    // they are held in registers, so an entry costs no chain of LDS reads)
    uint32_t lim[CO3_LUT_BITS_MAX + 1];
#pragma unroll
    for (uint32_t l = 1; l <= CO3_LUT_BITS_MAX; ++l) lim[l] = l <= lut_bits ? limit_s[l] : 0xffffffffu;
    for (uint32_t i = tid; i < (1u << lut_bits); i += HB_BLOCK) {
        uint32_t l = 1;
#pragma unroll
        for (uint32_t j = 1; j <= CO3_LUT_BITS_MAX; ++j) l += i >= lim[j] ? 1u : 0u;
        uint16_t entry = 0;
        if (l <= lut_bits) {
            uint32_t off = (i >> (lut_bits - l)) - (uint32_t)first_s[l];
            entry = (uint16_t)((l << 8) | sorted_s[base_s[l] + off]);
        }
        out->lut[i] = entry;
    }
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
