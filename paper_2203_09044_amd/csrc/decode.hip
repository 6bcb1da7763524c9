// Parameter-server side of Algorithm 1: chunk-indexed Huffman decoding with an LDS lookup
// table (one lane per chunk), and the average of the reconstructed user gradients.
#include "co3_dev.h"
#include "kernels.h"

#define DE_BLOCK 1024

__device__ __forceinline__ const Co3Code *dcode_of(const void *codes, int u)
{
    return reinterpret_cast<const Co3Code *>(reinterpret_cast<const char *>(codes) + (size_t)u * CO3_CODE_BYTES);
}

// ------------------------------------------------------------------------------------------
// Per-lane stream window in LDS.  The stream is read in 16-byte blocks (4 pieces of 32 bits; piece q
// holds stream bits [32q, 32q+32), first bit on top; in memory the words are little-endian u64, so
// the two pieces of a word are swapped).  Each lane keeps the 4 most recent blocks of its chunk in
// a 16-dword ring, stored in descending piece order (piece q at ring index 16 - (q mod 16), and a
// copy of the piece with q mod 16 == 0 at index 0) so that pieces q+1 and q are ring entries j and
// j+1 of one two-address LDS read.  The rings of a wavefront are interleaved: entry j of lane l is
// dword j*64 + l of the wavefront's area, so the bank of an access depends on the lane only and
// lanes at different ring positions never conflict.  Blocks are requested one run (16 symbols, 32
// with the two-symbol table) ahead of their use, at a cadence that is the same for all lanes of the
// wavefront, so the global-load latency hides behind the decoding of the previous run.
// ------------------------------------------------------------------------------------------
#define RING_ROWS 17
#define RING_ROW_DW CO3_WAVE     // dwords between consecutive ring entries of one lane
#define DE_GROUP 16          // symbols per run: one ring refill point, one 16-byte store
#define DE_MISS_LEN 255u     // length field of a table entry that does not resolve a symbol
#define DE_PAIR_BITS 12      // prefix length of the two-symbol table used for alphabets of at most 16 symbols
enum { DE_SHORT = 0, DE_LONG = 1, DE_PAIRS = 2 };   // fast-path variants of decode_range

struct LaneStream {
    const uint4 *blocks;   // the user's stream as 16-byte blocks
    int64_t nblocks;       // blocks inside the buffer; beyond read as zeros
    int64_t base_blk;      // absolute index of relative block 0 (the block holding the chunk start)
    uint32_t *slot;        // this lane's ring in LDS
    uint32_t rel;          // current bit position relative to block base_blk
    uint32_t loaded;       // relative blocks [loaded-4, loaded) are in the ring
    uint32_t nfly;         // blocks requested beyond `loaded`: fl0 holds block loaded, fl1 block loaded+1
    uint4 fl0, fl1;

    __device__ __forceinline__ uint4 fetch(uint32_t relblk) const
    {
        int64_t b = base_blk + relblk;
        return (b >= 0 && b < nblocks) ? blocks[b] : make_uint4(0u, 0u, 0u, 0u);
    }
    __device__ __forceinline__ void put(uint32_t relblk, uint4 v)
    {
        uint32_t top = 16u - (relblk & 3u) * 4u;   // ring index of the block's first piece
        slot[(top - 3) * RING_ROW_DW] = v.z;
        slot[(top - 2) * RING_ROW_DW] = v.w;
        slot[(top - 1) * RING_ROW_DW] = v.x;
        slot[top * RING_ROW_DW] = v.y;
        if (top == 16u) slot[0] = v.y;
    }
    __device__ __forceinline__ void land()
    {
        if (nfly >= 1u) put(loaded, fl0);
        if (nfly == 2u) put(loaded + 1u, fl1);
        loaded += nfly;
        nfly = 0;
    }
    // make pieces [.., need_dw) resident (synchronous; only used off the fast path).  Callers ask for
    // at most block cur+2, so the block overwritten (loaded-4) always lies behind the position.
    __device__ __forceinline__ void ensure(uint32_t need_dw)
    {
        land();
        while (loaded * 4u < need_dw) {
            put(loaded, fetch(loaded));
            ++loaded;
        }
    }
    __device__ __forceinline__ void open(uint64_t p0)
    {
        base_blk = (int64_t)(p0 >> 7);
        rel = (uint32_t)(p0 & 127u);
        nfly = 0;
        uint4 a = fetch(0), b = fetch(1), c = fetch(2), d = fetch(3);
        put(0, a);
        put(1, b);
        put(2, c);
        put(3, d);
        loaded = 4;
    }
    // Start of a run of DE_GROUP symbols: what was requested at the previous boundary enters the ring,
    // and up to two further blocks are requested so that four blocks from the current one on are
    // resident or on their way.  The blocks they will replace lie behind the position.
    __device__ __forceinline__ void group_boundary()
    {
        land();
        const uint32_t want = (rel >> 7) + 4u;
        if (loaded < want) {
            fl0 = fetch(loaded);
            nfly = 1;
            if (loaded + 1u < want) {
                fl1 = fetch(loaded + 1u);
                nfly = 2;
            }
        }
    }
    __device__ __forceinline__ uint64_t pos() const { return ((uint64_t)base_blk << 7) + rel; }
    // the 32 stream bits at the current position
    __device__ __forceinline__ uint32_t peek32() const
    {
        const uint32_t *pc = slot + (~(rel >> 5) & 15u) * RING_ROW_DW;
        uint64_t two = ((uint64_t)pc[RING_ROW_DW] << 32) | (uint64_t)pc[0];
        return (uint32_t)((two << (rel & 31u)) >> 32);
    }
    __device__ __forceinline__ uint32_t piece(uint32_t d) const { return slot[(16u - (d & 15u)) * RING_ROW_DW]; }
    __device__ __forceinline__ uint64_t peek64()
    {
        uint32_t d = rel >> 5, o = rel & 31u;
        ensure(d + 3u);
        uint64_t hi = ((uint64_t)piece(d) << 32) | (uint64_t)piece(d + 1u);
        uint64_t lo = (uint64_t)piece(d + 2u);
        return o ? ((hi << o) | (lo >> (32u - o))) : hi;
    }
};

// LDS-resident decoder tables of one code.  BITS: longest prefix the lookup table resolves.  The code
// blob stores a table of at most CO3_LUT_BITS_MAX bits; a workgroup that has LDS to spare widens it
// (DE_WIDE_BITS) while loading, so that fewer codewords take the canonical search.
#define DE_WIDE_BITS 14
template <int BITS>
struct DecTablesT {
    static constexpr int kBits = BITS;
    uint16_t lut[1 << BITS];
    uint64_t first_code[65];
    uint16_t count[66];
    uint16_t base[66];
    uint8_t sorted[256];
    uint64_t lim_incl[65];   // largest 64-bit window (codeword left-aligned, ones below) of a codeword of length <= l
    uint32_t maxlen, lut_bits;
};
typedef DecTablesT<CO3_LUT_BITS_MAX> DecTables;

template <class Tables>
__device__ __forceinline__ void load_tables(Tables &t, const Co3Code *cd)
{
    constexpr uint32_t BITS = Tables::kBits;
    const uint32_t lb = cd->lut_bits > CO3_LUT_BITS_MAX ? CO3_LUT_BITS_MAX : (cd->lut_bits < 1 ? 1 : cd->lut_bits);
    const uint32_t ml = cd->maxlen > 64 ? 64 : cd->maxlen;
    // table prefix here: the stored one, widened up to BITS when the code has longer codewords
    const uint32_t nb = (BITS > CO3_LUT_BITS_MAX && ml > lb) ? (ml < BITS ? ml : BITS) : lb;
    for (int i = threadIdx.x; i < 65; i += blockDim.x) t.first_code[i] = cd->first_code[i];
    for (int i = threadIdx.x; i < 66; i += blockDim.x) {
        t.count[i] = cd->count[i];
        t.base[i] = cd->base[i];
    }
    for (int i = threadIdx.x; i < 256; i += blockDim.x) t.sorted[i] = cd->sorted[i];
    if (threadIdx.x == 0) {
        t.maxlen = ml;
        t.lut_bits = nb;
    }
    if (nb == lb) {
        for (uint32_t i = threadIdx.x; i < (1u << lb); i += blockDim.x) {
            uint16_t e = cd->lut[i];
            t.lut[i] = (e >> 8) ? e : (uint16_t)(DE_MISS_LEN << 8);   // miss: longer than the prefix, or invalid
        }
        __syncthreads();
    } else {
        __syncthreads();                 // the canonical tables are read below
        for (uint32_t i = threadIdx.x; i < (1u << nb); i += blockDim.x) {
            uint32_t e = cd->lut[i >> (nb - lb)];
            if ((e >> 8) == 0u) {        // not resolved by the stored prefix: lengths lb+1 .. nb by the canonical rule
                e = DE_MISS_LEN << 8;
                for (uint32_t l = lb + 1; l <= nb; ++l) {
                    const uint64_t off = (uint64_t)(i >> (nb - l)) - t.first_code[l];
                    if (off < (uint64_t)t.count[l]) {
                        e = (l << 8) | t.sorted[(t.base[l] + (uint32_t)off) & 255u];
                        break;
                    }
                }
            }
            t.lut[i] = (uint16_t)e;
        }
        __syncthreads();
    }
    if (t.maxlen > t.lut_bits) {      // only codes with codewords beyond the table prefix use the limits
        for (int l = threadIdx.x; l < 65; l += blockDim.x) {
            int j = l;
            while (j >= 1 && t.count[j] == 0) --j;     // canonical order: shorter codewords are numerically below
            uint64_t lim = 0;
            if (j >= 1) {
                const uint64_t last = t.first_code[j] + t.count[j] - 1;
                lim = j == 64 ? last : (last << (64 - j)) | ((~0ull) >> j);
            }
            t.lim_incl[l] = lim;
        }
    }
}

// Two-symbol table for small alphabets (most pairs of codewords fit DE_PAIR_BITS bits there): entry i
// describes the stream that starts with the DE_PAIR_BITS-bit prefix i.
//   bits 0..7 first symbol, 8..15 second symbol, 16..23 length of the first codeword (DE_MISS_LEN when
//   the prefix does not resolve it), 24..31 length of both codewords together, 0 when the prefix does
//   not hold the whole second codeword.
// NIB (symbols of at most four bits): both symbols share the low byte instead, the second one in its
// upper half, the form in which the averaging workspace stores them.
// The second codeword is looked up with the bits after the first one, zero-filled: a codeword that
// ends inside the prefix is determined by its own bits alone (prefix-free code).
template <bool NIB>
__device__ __forceinline__ void build_pairs(const DecTables &t, uint32_t *pairs)
{
    const uint32_t down = DE_PAIR_BITS - t.lut_bits;
    for (uint32_t i = threadIdx.x; i < (1u << DE_PAIR_BITS); i += blockDim.x) {
        const uint32_t e1 = t.lut[i >> down];
        const uint32_t l1 = e1 >> 8;
        uint32_t entry = DE_MISS_LEN << 16;
        if (l1 != DE_MISS_LEN) {
            entry = (e1 & 0xffu) | (l1 << 16);
            const uint32_t i2 = (i << l1) & ((1u << DE_PAIR_BITS) - 1u);
            const uint32_t e2 = t.lut[i2 >> down];
            const uint32_t l2 = e2 >> 8;
            if (l2 != DE_MISS_LEN && l1 + l2 <= DE_PAIR_BITS)
                entry |= ((e2 & 0xffu) << (NIB ? 4 : 8)) | ((l1 + l2) << 24);
        }
        pairs[i] = entry;
    }
}

// Canonical decoding of a codeword longer than the table prefix: the first length l whose l-bit
// prefix lies within that length's codeword range.  Returns the length, 0 if there is none.
template <class Tables>
__device__ __forceinline__ int decode_long(const Tables &t, uint64_t window, uint32_t *sym)
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

// Careful decoding of `count` <= 16 symbols (any codeword length, any stream content): used for runs
// that the fast path could not vouch for and for the ragged end of a chunk.  Leaves blocks
// cur .. cur+2 resident.  Symbols are returned 4 per word, first in the lowest byte.
template <class Tables>
__device__ __forceinline__ void decode_run_careful(const Tables &t, LaneStream &ls, int shift, int count, bool &ok,
                                                   uint32_t w[4])
{
    w[0] = w[1] = w[2] = w[3] = 0;
    for (int k = 0; k < count; ++k) {
        ls.ensure((ls.rel >> 5) + 2u);
        uint32_t e = t.lut[ls.peek32() >> shift];
        uint32_t l = e >> 8, s = e & 0xffu;
        if (l == DE_MISS_LEN) {
            l = (uint32_t)decode_long(t, ls.peek64(), &s);
            if (l == 0) {
                ok = false;
                l = 1;
                s = 0;
            }
        }
        ls.rel += l;
        uint32_t sh = s << (8 * (k & 3));
        if ((k >> 2) == 0) w[0] |= sh;
        else if ((k >> 2) == 1) w[1] |= sh;
        else if ((k >> 2) == 2) w[2] |= sh;
        else w[3] |= sh;
    }
    ls.ensure(((ls.rel >> 7) + 3u) * 4u);
}

// Two-symbol entry e read at position m holds only its first codeword: the entry completed with the
// second codeword from a lookup of its own (the combined length in the top byte).
template <bool NIB>
__device__ __forceinline__ uint32_t pair_second(const LaneStream &ls, const uint32_t *pairs, uint32_t e, uint32_t m,
                                                bool &bad)
{
    const uint32_t l1 = (e >> 16) & 0xffu;
    if (l1 == DE_MISS_LEN) {     // not even the first codeword: the careful path takes the run
        bad = true;
        return 2u << 24;
    }
    const uint32_t m1 = m - l1;
    const uint32_t *pc1 = ls.slot + ((m1 >> 5) & 15u) * RING_ROW_DW;
    const uint32_t e2 = pairs[__builtin_amdgcn_alignbit(pc1[RING_ROW_DW], pc1[0], m1) >> (32 - DE_PAIR_BITS)];
    uint32_t l2 = (e2 >> 16) & 0xffu;
    if (l2 == DE_MISS_LEN) {
        bad = true;
        l2 = 1u;
    }
    return (e & 0xffu) | ((e2 & 0xffu) << (NIB ? 4 : 8)) | ((l1 + l2) << 24);
}

// One lane decodes symbols [i0, i1) of its chunk; the stream is open at symbol i0.  Symbols leave in
// runs of 16: run r is stored at out + r * run_step (run_step = 16 gives the plain contiguous layout;
// the tiled layout used between decoding and averaging interleaves the runs of the 64 chunks of a
// wavefront so that each store instruction of the wavefront covers one contiguous KiB).  A range
// that does not start or end on a run boundary (tensor boundaries with one code per tensor, the end
// of the vector) takes the careful path for the partial runs and stores them byte by byte.
//
// The fast path decodes a run without a residency check per symbol and validates it afterwards:
// every window it read must lie inside the blocks that were resident when the run started, and
// every window must have started a codeword.  Otherwise the run is decoded again by the careful
// path from the saved position.  Codewords longer than the table prefix are resolved in place by a
// canonical search (the lengths' upper limits are ordered), in a branch the wavefront skips when
// no lane needs it.
//
// DE_SHORT is the instance for codes whose longest codeword fits the table prefix: there a miss can
// only come from an invalid stream; it advances by DE_MISS_LEN, more than 16 hits can, which the
// validation catches.  DE_PAIRS reads the two-symbol table `pairs`: one lookup per two symbols and one
// refill point per 32 symbols (with at most four bits per symbol on average the blocks requested at one
// boundary cover the symbols up to the next one); a lookup whose prefix does not hold both codewords
// takes the second one from a lookup of its own (in a branch the wavefront skips when no lane needs
// it), and a codeword longer than the prefix sends the run to the careful path.
template <int MODE, class Tables>
__device__ __forceinline__ void decode_range(const Tables &t, LaneStream &ls, int i0, int i1, uint8_t *out,
                                             int64_t run_step, bool &ok, const uint32_t *pairs = nullptr)
{
    static_assert(DE_GROUP * Tables::kBits < DE_MISS_LEN, "a miss must advance more than a run of hits can");
    constexpr bool LONG = MODE == DE_LONG;
    const int shift = 32 - (int)t.lut_bits;
    int i = i0;
    // cnt < 16 symbols from symbol i on, inside one run
    auto partial = [&](int cnt) {
        ls.group_boundary();
        uint32_t w[4];
        decode_run_careful(t, ls, shift, cnt, ok, w);
        uint8_t *dst = out + (int64_t)(i >> 4) * run_step + (i & 15);
        for (int k = 0; k < cnt; ++k) {
            uint32_t word = (k >> 2) == 0 ? w[0] : (k >> 2) == 1 ? w[1] : (k >> 2) == 2 ? w[2] : w[3];
            dst[k] = (uint8_t)(word >> (8 * (k & 3)));
        }
        i += cnt;
    };
    if ((i & 15) != 0 && i < i1) partial(16 - (i & 15) < i1 - i ? 16 - (i & 15) : i1 - i);
    if (MODE == DE_PAIRS) {
#pragma unroll 1
        for (; i + 2 * DE_GROUP <= i1; i += 2 * DE_GROUP) {
            ls.group_boundary();
            const uint32_t rel0 = ls.rel;
            uint32_t w[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
            uint32_t m = 0u - rel0;
            bool bad = false;
#pragma unroll
            for (int b = 0; b < DE_GROUP; ++b) {
                const uint32_t *pc = ls.slot + ((m >> 5) & 15u) * RING_ROW_DW;
                const uint32_t win = __builtin_amdgcn_alignbit(pc[RING_ROW_DW], pc[0], m);
                uint32_t e = pairs[win >> (32 - DE_PAIR_BITS)];
                if ((e >> 24) == 0u) e = pair_second<false>(ls, pairs, e, m, bad);
                m -= e >> 24;
                w[b >> 1] = __builtin_amdgcn_alignbit(e, w[b >> 1], 16);
            }
            ls.rel = 0u - m;
            if (bad || ls.rel + 64u > ls.loaded * 128u) {   // rare
                ls.rel = rel0;
                decode_run_careful(t, ls, shift, DE_GROUP, ok, w);
                decode_run_careful(t, ls, shift, DE_GROUP, ok, w + 4);
            }
            uint8_t *dst = out + (int64_t)(i >> 4) * run_step;
            *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            *reinterpret_cast<uint4 *>(dst + run_step) = make_uint4(w[4], w[5], w[6], w[7]);
        }
    }
#pragma unroll 1
    for (; i + DE_GROUP <= i1; i += DE_GROUP) {
        ls.group_boundary();
        const uint32_t rel0 = ls.rel;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        // Work with the negated position m = -rel.  The window of 32 stream bits at rel is
        // ({piece d, piece d+1} >> (m mod 32)) with d = (rel - 1) / 32, whose ring index is
        // bits 5..8 of m: one field extract, one two-address LDS read, one funnel shift.
        uint32_t m = 0u - rel0;
        bool bad = false;
        if (MODE == DE_PAIRS) {
#pragma unroll
            for (int b = 0; b < DE_GROUP / 2; ++b) {
                const uint32_t *pc = ls.slot + ((m >> 5) & 15u) * RING_ROW_DW;
                const uint32_t win = __builtin_amdgcn_alignbit(pc[RING_ROW_DW], pc[0], m);
                uint32_t e = pairs[win >> (32 - DE_PAIR_BITS)];
                if ((e >> 24) == 0u) e = pair_second<false>(ls, pairs, e, m, bad);   // rare
                m -= e >> 24;
                w[b >> 1] = __builtin_amdgcn_alignbit(e, w[b >> 1], 16);
            }
        } else {
#pragma unroll
        for (int b = 0; b < DE_GROUP; ++b) {
            const uint32_t row = (m >> 5) & 15u;
            const uint32_t *pc = ls.slot + row * RING_ROW_DW;
            const uint32_t d0 = pc[0];
            uint32_t win = __builtin_amdgcn_alignbit(pc[RING_ROW_DW], d0, m);
            uint32_t e = t.lut[win >> shift];
            if (LONG && (e >> 8) == DE_MISS_LEN) {
                // Codeword longer than the table prefix (skipped by the wavefront when no lane is here):
                // 64-bit window, then the first length whose largest left-aligned codeword is not below it.
                const uint32_t d2 = ls.slot[((row - 1u) & 15u) * RING_ROW_DW];
                const uint64_t w64 = ((uint64_t)win << 32) | (uint64_t)__builtin_amdgcn_alignbit(d0, d2, m);
                // (the limits do not decrease with the length and stay put beyond the longest codeword, so
                // counting the limits below the window gives the length; nearly all long codewords end
                // within four bits of the prefix: those limits are compared without a loop)
                const uint32_t l0 = t.lut_bits + 1u;
                uint32_t l = l0;
#pragma unroll
                for (uint32_t k = 0; k < 4u; ++k) l += w64 > t.lim_incl[l0 + k] ? 1u : 0u;
                if (l == l0 + 4u)
                    for (uint32_t j = l0 + 4u; j < t.maxlen; ++j) l += w64 > t.lim_incl[j] ? 1u : 0u;
                const uint64_t off = (w64 >> (64u - l)) - t.first_code[l];
                if (off < (uint64_t)t.count[l]) {
                    e = (l << 8) | t.sorted[(t.base[l] + (uint32_t)off) & 255u];
                } else {          // no codeword starts here
                    bad = true;
                    e = 1u << 8;
                }
            }
            m -= e >> 8;
            w[b >> 2] = __builtin_amdgcn_alignbit(e, w[b >> 2], 8);
        }
        }
        ls.rel = 0u - m;
        // every window read above (up to three dwords from the current one) must have been resident
        if (MODE == DE_LONG    ? (bad || ls.rel + 96u > ls.loaded * 128u)
            : MODE == DE_PAIRS ? (bad || ls.rel + 64u > ls.loaded * 128u)
                               : (ls.rel - rel0 > DE_GROUP * Tables::kBits ||
                                  ls.rel + 64u > ls.loaded * 128u)) {   // rare
            ls.rel = rel0;
            decode_run_careful(t, ls, shift, DE_GROUP, ok, w);
        }
        *reinterpret_cast<uint4 *>(out + (int64_t)(i >> 4) * run_step) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (i < i1) partial(i1 - i);
}

// A whole chunk of an alphabet of at most 16 symbols, written in the packed form of the averaging
// workspace: two symbols per byte (the earlier one in the low half), 32 symbols per 16-byte store, run r
// of 32 symbols at out + r * run_step.  One refill point per 32 symbols: with at most four bits per
// symbol on average the blocks requested at one boundary cover the symbols up to the next one.
__device__ __forceinline__ void decode_chunk_packed(const DecTables &t, LaneStream &ls, int nsym, uint8_t *out,
                                                    int64_t run_step, bool &ok, const uint32_t *pairs)
{
    const int shift = 32 - (int)t.lut_bits;
    // cnt <= 32 symbols by the careful path, packed; the rest of the 16 bytes is zero
    auto careful = [&](int cnt, uint32_t w[4]) {
        uint32_t b[8];
        decode_run_careful(t, ls, shift, cnt < DE_GROUP ? cnt : DE_GROUP, ok, b);
        if (cnt > DE_GROUP) decode_run_careful(t, ls, shift, cnt - DE_GROUP, ok, b + 4);
        else b[4] = b[5] = b[6] = b[7] = 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) {      // bytes 0x0d0c0b0a, 0x0h0g0f0e -> nibbles 0xhgfedcba
            const uint32_t lo = b[2 * k], hi = b[2 * k + 1];
            const uint32_t l2 = (lo | (lo >> 4)) & 0x00ff00ffu, h2 = (hi | (hi >> 4)) & 0x00ff00ffu;
            w[k] = ((l2 | (l2 >> 8)) & 0xffffu) | (((h2 | (h2 >> 8)) & 0xffffu) << 16);
        }
    };
    int i = 0;
#pragma unroll 1
    for (; i + 2 * DE_GROUP <= nsym; i += 2 * DE_GROUP) {
        ls.group_boundary();
        const uint32_t rel0 = ls.rel;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        uint32_t m = 0u - rel0;
        bool bad = false;
#pragma unroll
        for (int b = 0; b < DE_GROUP; ++b) {
            const uint32_t *pc = ls.slot + ((m >> 5) & 15u) * RING_ROW_DW;
            const uint32_t win = __builtin_amdgcn_alignbit(pc[RING_ROW_DW], pc[0], m);
            uint32_t e = pairs[win >> (32 - DE_PAIR_BITS)];
            if ((e >> 24) == 0u) e = pair_second<true>(ls, pairs, e, m, bad);   // rare
            m -= e >> 24;
            w[b >> 2] = __builtin_amdgcn_alignbit(e, w[b >> 2], 8);
        }
        ls.rel = 0u - m;
        if (bad || ls.rel + 64u > ls.loaded * 128u) {   // rare: see decode_range
            ls.rel = rel0;
            careful(2 * DE_GROUP, w);
        }
        *reinterpret_cast<uint4 *>(out + (int64_t)(i >> 5) * run_step) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (i < nsym) {                        // ragged end of the vector
        ls.group_boundary();
        uint32_t w[4];
        careful(nsym - i, w);
        *reinterpret_cast<uint4 *>(out + (int64_t)(i >> 5) * run_step) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// TILED = false: sym_out is [U][stride] symbols in order.  TILED = true: sym_out is the averaging
// workspace, [U][tiles][chunk_syms/16][64 lanes][16 symbols] with tile = 64 consecutive chunks.
// PAIRS: the workgroup also builds the two-symbol table (launched for alphabets of at most 16
// symbols and chunks of at least 32); with TILED the workspace then holds two symbols per byte,
// [U][tiles][chunk_syms/32][64 lanes][32 symbols in 16 bytes].
template <bool TILED, bool PAIRS>
__global__ __launch_bounds__(DE_BLOCK) void k_decode(const uint64_t *__restrict__ words, int64_t cap_words,
                                                      const uint64_t *__restrict__ chunk_bitoff, int chunk_syms,
                                                      int64_t nchunks, const void *__restrict__ codes,
                                                      int code_per_user, int64_t n, uint8_t *__restrict__ sym_out,
                                                      int64_t stride, int32_t *status)
{
    const int u = blockIdx.y;
    // tables first: their LDS offsets then fit the immediate field of the read instructions
    __shared__ struct {
        uint32_t pairs[PAIRS ? (1 << DE_PAIR_BITS) : 1];
        DecTablesT<PAIRS ? CO3_LUT_BITS_MAX : DE_WIDE_BITS> t;   // one symbol per lookup: the widened table
        alignas(256) uint32_t ring[DE_BLOCK * RING_ROWS];   // a multiple of the ring row: row offsets stay immediates
    } lds;
    auto &t = lds.t;
    uint32_t *const ring = lds.ring;
    uint32_t *const pairs = lds.pairs;

    // The chunk's stream position and its first blocks are requested before the tables are loaded, so
    // that the three memory latencies at the start of a workgroup overlap.
    const int64_t c = (int64_t)blockIdx.x * DE_BLOCK + threadIdx.x;
    const bool active = c < nchunks;
    const uint64_t *off = chunk_bitoff + (int64_t)u * (nchunks + 1);
    const uint64_t p0 = active ? off[c] : 0, p1 = active ? off[c + 1] : 0;
    LaneStream ls;
    ls.blocks = reinterpret_cast<const uint4 *>(words + (int64_t)u * cap_words);
    ls.nblocks = cap_words / 2;
    ls.slot = ring + (threadIdx.x / CO3_WAVE) * (RING_ROWS * RING_ROW_DW) + (threadIdx.x & (CO3_WAVE - 1));
    if (active) ls.open(p0);
    load_tables(t, dcode_of(codes, code_per_user ? u : 0));        // else one code shared by all users
    __syncthreads();
    if constexpr (PAIRS) {
        build_pairs<TILED>(t, pairs);
        __syncthreads();
    }
    if (!active) return;

    int64_t first = c * chunk_syms;
    int nsym = (int)(n - first < chunk_syms ? n - first : chunk_syms);
    uint8_t *out;
    int64_t run_step;
    if (TILED) {
        const int64_t tile_bytes = (int64_t)CO3_WAVE * (PAIRS ? chunk_syms >> 1 : chunk_syms);
        out = sym_out + (int64_t)u * stride + (c >> 6) * tile_bytes + (c & 63) * 16;
        run_step = CO3_WAVE * 16;
    } else {
        out = sym_out + (int64_t)u * stride + first;
        run_step = 16;
    }
    bool ok = true;
    if constexpr (PAIRS && TILED) decode_chunk_packed(t, ls, nsym, out, run_step, ok, pairs);
    else if constexpr (PAIRS) decode_range<DE_PAIRS>(t, ls, 0, nsym, out, run_step, ok, pairs);
    else if (t.maxlen > t.lut_bits) decode_range<DE_LONG>(t, ls, 0, nsym, out, run_step, ok);
    else decode_range<DE_SHORT>(t, ls, 0, nsym, out, run_step, ok);
    ls.land();
    if (!(ok && ls.pos() == p1)) co3_raise(status, CO3_EBADSTREAM);
}

// Decompression with one code per tensor shared by all users (Sec. III (ii) as stated).  The workgroup
// walks the tensors of its range of elements with the tables of four neighbouring tensors resident
// (tensor s in slot s mod 4): a lane decodes the part of its chunk that lies in the tensor at its
// position as soon as that tensor's tables are there, so the chunks on both sides of a tensor
// boundary are decoded at the same time, each lane reading the table of its own tensor; a chunk that
// straddles tensors goes on into the next tensor while that tensor's tables are in the window.  Lanes whose tensor is more than three tensors away
// from the first one of the range wait for the window: tensors much smaller than a workgroup's range
// (512 chunks) are better given a code together with a neighbour.
#define DL_BLOCK 512
#define DL_SLOTS 4

template <bool TILED>
__global__ __launch_bounds__(DL_BLOCK) void k_decode_layers(const uint64_t *__restrict__ words, int64_t cap_words,
                                                             const uint64_t *__restrict__ chunk_bitoff, int chunk_syms,
                                                             int64_t nchunks, const void *__restrict__ codes,
                                                             const int64_t *__restrict__ seg_off, int nseg, int64_t n,
                                                             uint8_t *__restrict__ sym_out, int64_t stride,
                                                             int32_t *status)
{
    const int u = blockIdx.y;
    __shared__ DecTables t[DL_SLOTS];
    __shared__ uint32_t ring[DL_BLOCK * RING_ROWS];
    if (threadIdx.x < DL_SLOTS) {
        t[threadIdx.x].maxlen = 0;
        t[threadIdx.x].lut_bits = 1;
    }

    const int64_t c = (int64_t)blockIdx.x * DL_BLOCK + threadIdx.x;
    const bool active = c < nchunks;
    const uint64_t *off = chunk_bitoff + (int64_t)u * (nchunks + 1);
    LaneStream ls;
    ls.blocks = reinterpret_cast<const uint4 *>(words + (int64_t)u * cap_words);
    ls.nblocks = cap_words / 2;
    ls.slot = ring + (threadIdx.x / CO3_WAVE) * (RING_ROWS * RING_ROW_DW) + (threadIdx.x & (CO3_WAVE - 1));
    const int64_t first = c * chunk_syms;
    const int nsym = active ? (int)(n - first < chunk_syms ? n - first : chunk_syms) : 0;
    uint8_t *out;
    int64_t run_step;
    if (TILED) {
        out = sym_out + (int64_t)u * stride + (c >> 6) * ((int64_t)CO3_WAVE * chunk_syms) + (c & 63) * 16;
        run_step = CO3_WAVE * 16;
    } else {
        out = sym_out + (int64_t)u * stride + first;
        run_step = 16;
    }
    // tensors touched by the workgroup's range of elements (uniform)
    const int64_t b_first = (int64_t)blockIdx.x * DL_BLOCK * chunk_syms;
    int64_t b_last = b_first + (int64_t)DL_BLOCK * chunk_syms;
    b_last = (b_last < n ? b_last : n) - 1;
    const int b_lo = co3_find_seg(seg_off, nseg, b_first), b_hi = co3_find_seg(seg_off, nseg, b_last);

    bool ok = true;
    int cur = 0;                                                        // next symbol of the chunk to decode
    int cur_seg = nsym > 0 ? co3_find_seg(seg_off, nseg, first) : -1;   // the tensor that holds it
    if (nsym > 0) ls.open(off[c]);
    for (int sg = b_lo; sg <= b_hi; ++sg) {
        __syncthreads();                 // nobody reads the slot that is replaced any more
        if (sg == b_lo) {
            for (int k = 0; k < DL_SLOTS - 1 && sg + k <= b_hi; ++k)
                load_tables(t[(sg + k) & (DL_SLOTS - 1)], dcode_of(codes, sg + k));
        }
        if (sg + DL_SLOTS - 1 <= b_hi)
            load_tables(t[(sg + DL_SLOTS - 1) & (DL_SLOTS - 1)], dcode_of(codes, sg + DL_SLOTS - 1));
        __syncthreads();
        bool any_long = false;           // uniform
        for (int k = 0; k < DL_SLOTS; ++k) any_long |= t[k].maxlen > t[k].lut_bits;
        // a chunk that straddles tensors goes on at once while the next tensor's tables are in the window
        // (if it waited for the next step it would start its second part when all other lanes have finished
        // their whole chunks)
        while (cur < nsym && cur_seg >= sg && cur_seg < sg + DL_SLOTS) {
            const DecTables &tl = t[cur_seg & (DL_SLOTS - 1)];
            const int64_t seg_end = seg_off[cur_seg + 1] - first;
            const int i1 = seg_end < nsym ? (int)seg_end : nsym;
            if (i1 <= cur) break;        // boundaries that do not increase: the chunk stays unfinished and is reported
            if (any_long) decode_range<DE_LONG>(tl, ls, cur, i1, out, run_step, ok);
            else decode_range<DE_SHORT>(tl, ls, cur, i1, out, run_step, ok);
            cur = i1;
            if (cur < nsym) cur_seg = co3_find_seg(seg_off, nseg, first + cur);
        }
    }
    if (nsym > 0) {
        ls.land();
        ok = ok && cur == nsym && ls.pos() == off[c + 1];
    }
    if (!ok) co3_raise(status, CO3_EBADSTREAM);
}

// ---- average of the reconstructed gradients: users added in index order, one division -----
// Average from the tiled workspace: one thread owns the 16 bytes of one run, 16 consecutive elements
// (NIB, two symbols per byte: 32).  A workgroup of PT_WAVES wavefronts takes that many consecutive runs
// of one tile of 64 chunks.
#define PT_WAVES(NIB) ((NIB) ? 2 : 4)

// TABLE != 0 (one tensor, i.e. one anchor per user): the values of every user's symbols are computed
// once per block into LDS, and an element costs one LDS read and one add.  TABLE = 1 keeps all K
// values; TABLE = 2 (larger alphabets) keeps the K/2 magnitudes and applies the sign bit after the
// read, halving the LDS footprint.
template <int TABLE, bool NIB>
__global__ __launch_bounds__(PT_WAVES(NIB) * CO3_WAVE) void k_ps_sum_tiled(const uint8_t *__restrict__ symt, int64_t n, int U,
                                                            int64_t ws_stride, int chunk_syms, int64_t nruns,
                                                            const int32_t *__restrict__ anchor,
                                                            const float *__restrict__ scale,
                                                            const int64_t *__restrict__ seg_off_g, int nseg,
                                                            co3_fmt fmt, const float *acc_in, float divisor,
                                                            float *avg_out)
{
    constexpr int EPT = NIB ? 32 : 16;     // elements per thread
    constexpr int WAVES = PT_WAVES(NIB), PT_BLOCK = WAVES * CO3_WAVE;
    const FmtC fc(fmt);
    const int EM = fc.E + fc.M, M = fc.M, F = fc.F;
    const uint32_t cmask = (uint32_t)fc.codemax;
    const int runs_per_chunk = chunk_syms / EPT;
    // value of symbol s of user u in tensor sg; with multipliers (scale != NULL) the level is divided by
    // the user's multiplier, one fp32 rounding
    auto value = [&](uint32_t s, int u, int sg) -> float {
        const int e_min = anchor[(int64_t)u * nseg + sg] - F + 1;
        float v = __uint_as_float(__float_as_uint(co3_code_value(s & cmask, e_min, M)) | ((s >> EM) << 31));
        if (scale) v = v / scale[(int64_t)u * nseg + sg];
        return v;
    };
    // symbol k of the 16 bytes w
    auto symbol = [&](const uint32_t (&w)[4], int k) -> uint32_t {
        return NIB ? (w[k >> 3] >> (4 * (k & 7))) & 0xfu : (w[k >> 2] >> (8 * (k & 3))) & 0xffu;
    };
    __shared__ int64_t seg_cache[TABLE ? 1 : CO3_SEG_CACHE];     // TABLE: one tensor, nothing to look up
    const int64_t *seg_off = TABLE ? seg_off_g : co3_cache_segs(seg_off_g, nseg, seg_cache);
    extern __shared__ float value_of[];    // [U][K] or [U][K/2], TABLE only
    if (TABLE) {
        const int H = TABLE == 1 ? fc.K : fc.K >> 1;
        for (int j = threadIdx.x; j < U * H; j += PT_BLOCK) {
            const int u = j / H;
            value_of[j] = value((uint32_t)(j - u * H), u, 0);
        }
        __syncthreads();
    }
    // One block step covers one tile (64 chunks) x WAVES consecutive runs: each wavefront one run, each
    // lane one chunk (a chunk has a multiple of WAVES runs).  The WAVES * EPT results per chunk are
    // contiguous in the output; they pass through LDS so that every store instruction of a wavefront
    // writes 256 contiguous bytes.
    constexpr int ROW = WAVES * EPT;       // 64 elements in both layouts
    __shared__ float out_s[CO3_WAVE][ROW + 1];
    for (int64_t rb = (int64_t)blockIdx.x * PT_BLOCK; rb < nruns; rb += (int64_t)gridDim.x * PT_BLOCK) {
        // r enumerates (tile, run within chunk, lane) with the lane fastest: the workspace order
        const int64_t r = rb + threadIdx.x;
        const int lane = (int)(r & 63);
        const int wr = threadIdx.x >> 6;
        const int64_t q = r >> 6;
        const int run = (int)(q & (runs_per_chunk - 1));             // runs per chunk: a power of two
        const int64_t tile = q >> __builtin_ctz((unsigned)runs_per_chunk);
        const int64_t i0 = (tile * CO3_WAVE + lane) * chunk_syms + (int64_t)run * EPT;
        const uint8_t *src = symt + r * 16;
        // the sum starts at zero, or continues a sum over users before these (acc_in may be avg_out: every
        // element is read and written by the same workgroup, the reads first)
        float acc[EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) acc[k] = 0.f;
        if (acc_in && i0 < n) {
            if (i0 + EPT <= n) {
#pragma unroll
                for (int k = 0; k < EPT; k += 4) {
                    const float4 a = *reinterpret_cast<const float4 *>(acc_in + i0 + k);
                    acc[k] = a.x, acc[k + 1] = a.y, acc[k + 2] = a.z, acc[k + 3] = a.w;
                }
            } else {
#pragma unroll
                for (int k = 0; k < EPT; ++k)
                    if (i0 + k < n) acc[k] = acc_in[i0 + k];
            }
        }
        const int64_t i_first = i0 < n ? i0 : n - 1;       // lanes past the end compute on the last element's
        const int s_lo = TABLE ? 0 : co3_find_seg(seg_off, nseg, i_first);   // tensor and store nothing
        const int64_t i_last = i0 + EPT - 1 < n ? i0 + EPT - 1 : n - 1;
        const int s_hi = TABLE ? 0 : co3_find_seg(seg_off, nseg, i_last);
        if (i0 >= n) {
        } else if (TABLE) {
            for (int u = 0; u < U; ++u) {
                const float *vu = value_of + u * (TABLE == 1 ? fc.K : fc.K >> 1);
                uint4 v = ld_stream_u4(src + (int64_t)u * ws_stride);
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < EPT; ++k) {
                    const uint32_t sy = symbol(w, k);
                    if (TABLE == 1) acc[k] += vu[sy & ((uint32_t)fc.K - 1u)];
                    else acc[k] += __uint_as_float(__float_as_uint(vu[sy & cmask]) | (((sy >> EM) & 1u) << 31));
                }
            }
        } else if (s_lo == s_hi) {
            for (int u = 0; u < U; ++u) {
                const int e_min = anchor[(int64_t)u * nseg + s_lo] - F + 1;
                const float c = scale ? scale[(int64_t)u * nseg + s_lo] : 1.0f;
                uint4 v = *reinterpret_cast<const uint4 *>(src + (int64_t)u * ws_stride);
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < EPT; ++k) {
                    uint32_t s = symbol(w, k);
                    float val = co3_code_value(s & cmask, e_min, M);
                    val = __uint_as_float(__float_as_uint(val) | ((s >> EM) << 31));
                    acc[k] += scale ? val / c : val;
                }
            }
        } else {                           // the run straddles tensors: anchor per element
            for (int u = 0; u < U; ++u) {
                uint4 v = *reinterpret_cast<const uint4 *>(src + (int64_t)u * ws_stride);
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < EPT; ++k) {
                    int sg = co3_find_seg(seg_off, nseg, i0 + k < n ? i0 + k : n - 1);
                    acc[k] += value(symbol(w, k), u, sg);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < EPT; ++k) out_s[lane][wr * EPT + k] = divisor > 0.f ? acc[k] / divisor : acc[k];
        __syncthreads();
        const int64_t run0 = (int64_t)(run - wr) * EPT;      // first element (within a chunk) of the block's runs
#pragma unroll 4
        for (int j = 0; j < CO3_WAVE; j += WAVES) {
            const int idx = (j + wr) * CO3_WAVE + (threadIdx.x & 63);   // element of the [64][ROW] tile, row-major
            const int cc = idx / ROW, e = idx % ROW;
            const int64_t i = (tile * CO3_WAVE + cc) * chunk_syms + run0 + e;
            if (i < n) __builtin_nontemporal_store(out_s[cc][e], avg_out + i);   // not read again here
        }
        __syncthreads();
    }
}

// seg_off != NULL selects one code per tensor (codes[tensor], shared by the users) instead of codes[user]
hipError_t co3_launch_decode(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int chunk_syms,
                             const void *codes, const int64_t *seg_off, int nseg, int K, int64_t n, int U,
                             uint8_t *sym_out, int64_t stride, int tiled, int32_t *status, hipStream_t st)
{
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    if (nchunks <= 0) return hipSuccess;
    unsigned blocks = (unsigned)((nchunks + DE_BLOCK - 1) / DE_BLOCK);
    const unsigned lblocks = (unsigned)((nchunks + DL_BLOCK - 1) / DL_BLOCK);
#define CO3_DECODE_LAUNCH(T, P)                                                                                    \
    hipLaunchKernelGGL((k_decode<T, P>), dim3(blocks, U), dim3(DE_BLOCK), 0, st, words, cap_words, chunk_bitoff,   \
                       chunk_syms, nchunks, codes, code_per_user, n, sym_out, stride, status)
    Co3LaunchTimer tm(CO3_K_DECODE, st);
    // one code for everything, shared by the users: the per-user kernels with every user reading codes[0]
    const int code_per_user = seg_off == nullptr;
    if (seg_off && nseg == 1) seg_off = nullptr;
    if (seg_off && tiled)
        hipLaunchKernelGGL(k_decode_layers<true>, dim3(lblocks, U), dim3(DL_BLOCK), 0, st, words, cap_words,
                           chunk_bitoff, chunk_syms, nchunks, codes, seg_off, nseg, n, sym_out, stride, status);
    else if (seg_off)
        hipLaunchKernelGGL(k_decode_layers<false>, dim3(lblocks, U), dim3(DL_BLOCK), 0, st, words, cap_words,
                           chunk_bitoff, chunk_syms, nchunks, codes, seg_off, nseg, n, sym_out, stride, status);
    else if (co3_ws_packed(K, chunk_syms, 0)) {
        if (tiled) CO3_DECODE_LAUNCH(true, true);
        else CO3_DECODE_LAUNCH(false, true);
    } else {
        if (tiled) CO3_DECODE_LAUNCH(true, false);
        else CO3_DECODE_LAUNCH(false, false);
    }
#undef CO3_DECODE_LAUNCH
    return hipGetLastError();
}

hipError_t co3_launch_ps_sum_tiled(const uint8_t *symt, int64_t n, int U, int64_t ws_stride, int chunk_syms,
                                   const int32_t *anchor, const float *scale, const int64_t *seg_off, int nseg,
                                   co3_fmt fmt, int packed, const float *acc_in, float divisor, float *avg_out,
                                   hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    const int64_t ntiles = (nchunks + CO3_WAVE - 1) / CO3_WAVE;
    const int64_t nruns = ntiles * (chunk_syms >> (packed ? 5 : 4)) * CO3_WAVE;   // 16-byte pieces of one user
    const int threads = PT_WAVES(packed) * CO3_WAVE;
    int64_t b = (nruns + threads - 1) / threads;
    unsigned blocks = (unsigned)(b < 16384 ? b : 16384);
    Co3LaunchTimer tm(CO3_K_PS_SUM, st);
    const size_t full_bytes = (size_t)U * (size_t)(1 << (1 + fmt.exp_bits + fmt.mant_bits)) * sizeof(float);
#define CO3_SUM_LAUNCH(T, P, BYTES)                                                                                \
    hipLaunchKernelGGL((k_ps_sum_tiled<T, P>), dim3(blocks), dim3(threads), BYTES, st, symt, n, U, ws_stride,     \
                       chunk_syms, nruns, anchor, scale, seg_off, nseg, fmt, acc_in, divisor, avg_out)
    if (packed) {       // alphabets of at most 16 symbols: the full table is 64 bytes per user
        if (nseg == 1 && full_bytes <= 4096) CO3_SUM_LAUNCH(1, true, full_bytes);
        else CO3_SUM_LAUNCH(0, true, 0);
    } else if (nseg == 1 && full_bytes <= 4096) CO3_SUM_LAUNCH(1, false, full_bytes);
    else if (nseg == 1 && full_bytes / 2 <= 32768) CO3_SUM_LAUNCH(2, false, full_bytes / 2);
    else CO3_SUM_LAUNCH(0, false, 0);
#undef CO3_SUM_LAUNCH
    return hipGetLastError();
}
