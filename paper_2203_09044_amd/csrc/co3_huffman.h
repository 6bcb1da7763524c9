// Huffman code construction (Sec. III (ii)) by a group of NT lanes (a workgroup of 256, or one wavefront):
// code lengths by the two-queue merge, canonical codewords, and the decoder tables of the code blob, from
// K <= 256 integer weights.  Lane t of the group owns symbols t, t + NT, ...
#pragma once
#include "co3_dev.h"

struct Co3BuildLds {
    uint64_t key[256];          // (weight << 8 | symbol), inactive symbols sort last
    uint64_t node_w[512];       // weights of merged nodes (index >= nact)
    uint64_t leaf_q[256 + 4];
    uint64_t first_s[66];
    uint32_t cnt_s[66];
    uint32_t base_s[66];
    uint32_t limit_s[CO3_LUT_BITS_MAX + 2];
    uint32_t maxlen_s, nact_s;
    uint16_t parent[512];
    __attribute__((aligned(4))) uint8_t len_s[256];   // also read as words
    uint8_t sorted_s[256];
};

struct Co3BlockSync {
    __device__ __forceinline__ void operator()() const { __syncthreads(); }
};
struct Co3WaveSync {
    __device__ __forceinline__ void operator()() const { co3_wave_lds_sync(); }
};

#define CO3_PUB_VALID (1ull << 63)      // published table entries carry this bit (an entry is below 2^63)

// wt[j]: weight of symbol tid + j * NT.  out: the user's code blob.  pub (optional): K words in global
// memory that receive (codeword << 6 | length) | CO3_PUB_VALID of every symbol with a relaxed device-scope
// store, for readers inside the same kernel, as soon as the codewords are known.
template <int NT, class Sync>
__device__ __forceinline__ void co3_build_code_group(Co3BuildLds &L, const int tid, const uint32_t (&wt)[256 / NT],
                                                     const int K, Co3Code *out, uint64_t *pub, int32_t *status, Sync sync)
{
    constexpr int PER = 256 / NT;
    uint64_t mykey[PER];
    int mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int s = tid + j * NT;
        mykey[j] = wt[j] ? (((uint64_t)wt[j] << 8) | (uint64_t)s) : ~0ull;
        mine += wt[j] ? 1 : 0;
        L.key[s] = mykey[j];
        L.len_s[s] = 0;
        L.sorted_s[s] = 0;
    }
    for (int i = tid; i < 66; i += NT) {
        L.cnt_s[i] = 0;
        L.first_s[i] = 0;
        L.base_s[i] = 0;
    }
    if (tid == 0) {
        L.maxlen_s = 0;
        L.nact_s = 0;
    }
    sync();
    if (mine) atomicAdd(&L.nact_s, (uint32_t)mine);
    sync();
    const int nact = (int)L.nact_s;

    // leaves in (weight, symbol) order: every lane counts the keys below its own (all lanes read the
    // same entry at the same time, a broadcast) and stores its key at that position; the symbols without
    // a weight share one key and are ordered among themselves by their index
    {
        int below[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) below[j] = 0;
        for (int i = 0; i < K; ++i) {        // entries from K on hold the no-weight key and stay where they are
            const uint64_t ki = L.key[i];
#pragma unroll
            for (int j = 0; j < PER; ++j) below[j] += (ki < mykey[j] || (ki == mykey[j] && i < tid + j * NT)) ? 1 : 0;
        }
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (tid + j * NT >= K) below[j] = tid + j * NT;
        sync();
#pragma unroll
        for (int j = 0; j < PER; ++j) L.key[below[j]] = mykey[j];
        sync();
    }

    // two-queue merge: nodes 0..nact-1 are the sorted leaves, nact..2*nact-2 the merged nodes in
    // creation order; a leaf wins a weight tie against a merged node.
    // One lane runs the merge.  A step reads the two front entries of each queue and takes one of three
    // outcomes: two leaves (the second leaf is not above the first node), two nodes (the second node is
    // below the first leaf), or the first leaf with the first node (their order does not matter to the
    // sum or to the parent links).  Both queues are padded with an unreachable weight, so no bounds
    // test is needed; the node created by a step is written before the next step reads the fronts.
    const uint64_t INF = ~0ull;     // weights stay below 2^40, so INF never wins while a queue has entries
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int s = tid + j * NT;
        L.leaf_q[s] = s < nact ? (L.key[s] >> 8) : INF;
        L.node_w[s] = INF;
        L.node_w[256 + s] = INF;
    }
    if (tid < 4) L.leaf_q[256 + tid] = INF;
    sync();
    if (tid == 0 && nact >= 2) {
        int q1 = 0, q2 = nact;
        for (int next = nact; next < 2 * nact - 1; ++next) {
            const uint64_t L0 = L.leaf_q[q1], L1 = L.leaf_q[q1 + 1];
            const uint64_t N0 = L.node_w[q2], N1 = L.node_w[q2 + 1];
            uint64_t wsum;
            if (L1 <= N0) {
                wsum = L0 + L1;
                L.parent[q1] = (uint16_t)next;
                L.parent[q1 + 1] = (uint16_t)next;
                q1 += 2;
            } else if (N1 < L0) {
                wsum = N0 + N1;
                L.parent[q2] = (uint16_t)next;
                L.parent[q2 + 1] = (uint16_t)next;
                q2 += 2;
            } else {
                wsum = L0 + N0;
                L.parent[q1] = (uint16_t)next;
                L.parent[q2] = (uint16_t)next;
                ++q1;
                ++q2;
            }
            L.node_w[next] = wsum;
        }
    }
    sync();

    // code length = depth of the leaf
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int leaf = tid + j * NT;
        if (leaf < nact) {
            int depth;
            if (nact == 1) {
                depth = 1;
            } else {
                const int root = 2 * nact - 2;
                depth = 0;
                for (int v = leaf; v != root && depth < 255; v = L.parent[v]) ++depth;
            }
            const int s = (int)(L.key[leaf] & 0xffu);
            const int dl = depth > 64 ? 64 : depth;
            L.len_s[s] = (uint8_t)dl;
            atomicAdd(&L.cnt_s[dl], 1u);
            atomicMax(&L.maxlen_s, (uint32_t)depth);
        }
    }
    sync();
    const uint32_t maxlen = L.maxlen_s;
    if (tid == 0 && maxlen > CO3_MAX_CODE_LEN) co3_raise(status, CO3_EINVAL);

    // canonical numbering: first code of length l is sum_{j<l} count[j] << (l - j)
    for (int l = 1 + tid; l <= 64; l += NT) {
        uint64_t first = 0;
        uint32_t base = 0;
        for (int j = 1; j < l; ++j) {
            first += (uint64_t)L.cnt_s[j] << (l - j);
            base += L.cnt_s[j];
        }
        L.first_s[l] = first;
        L.base_s[l] = base;
    }
    sync();

#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int s = tid + j * NT;
        const uint32_t l = L.len_s[s];
        uint64_t enc = 0;
        if (l) {
            // symbols below this one with the same length, four length bytes per LDS word
            uint32_t rank = 0;
            const uint32_t *len_w = reinterpret_cast<const uint32_t *>(L.len_s);
            const uint32_t pat = l * 0x01010101u;
            for (int i = 0; i <= s >> 2; ++i) {
                uint32_t x = len_w[i] ^ pat;                       // zero bytes where the length matches
                if (i == s >> 2) x |= ~0u << (8 * (s & 3));        // only the symbols below this one
                const uint32_t z = ~(((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x | 0x7f7f7f7fu);   // 0x80 per zero byte
                rank += (uint32_t)__builtin_popcount(z);
            }
            const uint64_t code = L.first_s[l] + rank;
            L.sorted_s[L.base_s[l] + rank] = (uint8_t)s;
            enc = (code << 6) | (uint64_t)(l & 63u);
        }
        if (pub && s < K) __hip_atomic_store(pub + s, enc | CO3_PUB_VALID, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        out->len[s] = (uint8_t)l;
        out->enc[s] = enc;
    }
    sync();

    for (int i = tid; i < 65; i += NT) out->first_code[i] = L.first_s[i];
    for (int i = tid; i < 66; i += NT) {
        out->count[i] = (uint16_t)L.cnt_s[i];
        out->base[i] = (uint16_t)L.base_s[i];
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) out->sorted[tid + j * NT] = L.sorted_s[tid + j * NT];
    const uint32_t lut_bits = maxlen < 1 ? 1 : (maxlen > CO3_LUT_BITS_MAX ? CO3_LUT_BITS_MAX : maxlen);
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
    for (int l = 1 + tid; l <= (int)lut_bits; l += NT) {
        const uint64_t lim = (L.first_s[l] + L.cnt_s[l]) << (lut_bits - l);
        L.limit_s[l] = lim > (1ull << lut_bits) ? (1u << lut_bits) : (uint32_t)lim;
    }
    sync();
    // (the limits do not decrease with the length: counting the limits at or below i gives the length;
    // they are held in registers, so an entry costs no chain of LDS reads)
    uint32_t lim[CO3_LUT_BITS_MAX + 1];
#pragma unroll
    for (uint32_t l = 1; l <= CO3_LUT_BITS_MAX; ++l) lim[l] = l <= lut_bits ? L.limit_s[l] : 0xffffffffu;
    for (uint32_t i = tid; i < (1u << lut_bits); i += NT) {
        uint32_t l = 1;
#pragma unroll
        for (uint32_t j = 1; j <= CO3_LUT_BITS_MAX; ++j) l += i >= lim[j] ? 1u : 0u;
        uint16_t entry = 0;
        if (l <= lut_bits) {
            const uint32_t off = (i >> (lut_bits - l)) - (uint32_t)L.first_s[l];
            entry = (uint16_t)((l << 8) | L.sorted_s[L.base_s[l] + off]);
        }
        out->lut[i] = entry;
    }
}
