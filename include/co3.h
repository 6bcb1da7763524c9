/*
 * libco3 -- C ABI of the CO3 gradient codec hot path on one MI355X (gfx950).
 *
 * The calls follow one iteration of Algorithm 1 of "Convert, compress, correct":
 * on the user side error correction + fp conversion (co3_convert_ef), the symbol
 * statistics and the Huffman code (co3_histogram, co3_build_code), compression
 * (co3_encode); on the parameter-server side decompression (co3_decode) and
 * decompression + averaging over users (co3_ps_aggregate).  All U users of an
 * iteration are batched in every call.
 *
 * Conventions for every call below, unless its comment says otherwise:
 *   - every pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates or frees device memory and keeps no state between calls.  The
 *     exceptions, all process-wide: the fixed workspace of co3_encode_static, the
 *     poll limit set by co3_set_exchange_spin_limit (an atomic word), and, only
 *     while co3_timing_enable has switched it on, a pool of events for the
 *     per-kernel timer (not thread-safe: a diagnostic for single-threaded use);
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); the
 *     call only enqueues kernels on it and returns without waiting;
 *   - batched arrays are laid out [U][stride] with `stride` in elements (>= n, and
 *     a multiple of 16 when U > 1); float, symbol and word arrays must be 16-byte
 *     aligned, and cap_words (the per-user stride of the word array) must be even;
 *   - the return value is a host-side status: CO3_OK or a negative CO3_E* for
 *     arguments rejected before anything was launched;
 *   - conditions that only the device can see (capacity overrun, symbol without a
 *     code, inconsistent stream) are reported through `status`, a caller-owned
 *     device int32 that the caller zeroes once; kernels only ever lower it to a
 *     negative CO3_E* value (the smallest wins) and never write out of bounds.
 *     Read it with co3_poll_status.
 *
 * Format of the sign/exponent/mantissa representation (Sec. III (i)): 1 sign bit,
 * E exponent bits, M mantissa bits, K = 2^(1+E+M) <= 256 symbols; symbol byte =
 * sign << (E+M) | exponent field << M | mantissa field.  The exponent bias is an
 * integer anchor A per (user, segment): exponent field f >= 1 is binade
 * 2^(A - (2^E - 1) + f), field 0 holds the gradual-underflow levels (including 0),
 * there are no Inf/NaN codes, and the negative-zero pattern is never produced.
 *
 * Format of a compressed stream (Sec. II-B: h is an invertible variable-length
 * map; Sec. III (ii): element-wise Huffman): canonical Huffman codewords
 * concatenated most-significant bit first; stream bit p is bit 63 - (p mod 64) of
 * 64-bit word p / 64; the last word is zero padded.  chunk_bitoff[c] is the stream
 * position of symbol c * chunk_syms, chunk_bitoff[nchunks] the stream length,
 * nchunks = ceil(n / chunk_syms).  The wire header of a user is len[K] (the first K
 * bytes of its code blob), its anchors and n.
 */
#ifndef CO3_H
#define CO3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t exp_bits;  /* E >= 1 */
    int32_t mant_bits; /* M >= 0, 1 + E + M <= 8 */
} co3_fmt;

#define CO3_OK 0
#define CO3_EINVAL (-1)     /* bad argument (format, size, alignment, null pointer) */
#define CO3_ECAP (-2)       /* a stream would exceed cap_words; that user's stream is incomplete */
#define CO3_ENOCODE (-3)    /* a symbol to encode has no codeword (possible with model tables) */
#define CO3_EBADSTREAM (-4) /* decoder: a chunk did not end where the index says, or an invalid prefix */
#define CO3_EHIP (-5)       /* a HIP runtime call failed */
#define CO3_ETIMEOUT (-6)   /* a bounded wait inside a kernel ran out (co3_user_encode); results unspecified */

#define CO3_ANCHOR_GIVEN 0         /* anchor[] is an input */
#define CO3_ANCHOR_FROM_ABSMAX_G 1 /* anchor[] is an output: binade of max|g| per (user, segment) */

#define CO3_CODE_BYTES 12288 /* size of one user's code blob */

/* ---- helpers (host only, no GPU work) ---------------------------------- */

/* Human-readable name of a status code; never NULL. */
const char *co3_strerror(int32_t status);

/* Bytes of workspace co3_encode needs (per user one 64-bit partial sum per tile of 1024 symbols and
 * one per group of 16 tiles). */
size_t co3_encode_workspace_bytes(int64_t n, int32_t U);

/* Bytes of workspace co3_ps_aggregate needs (the decoded symbols of all users, whole tiles of
 * 64 chunks). */
size_t co3_ps_aggregate_workspace_bytes(int64_t n, int32_t U, int32_t chunk_syms);

/* Number of 64-bit words that always hold a stream coded with an empirical table built
 * from the very symbols being coded (Huffman is then no longer than the fixed-length
 * code): ceil(n * (1+E+M) / 64), rounded up to a multiple of 2. */
int64_t co3_cap_words_empirical(int64_t n, co3_fmt fmt);

/* Waits for `stream` and returns the device status word (CO3_OK if it is still 0),
 * or CO3_EHIP.  status_dev: device int32. */
int32_t co3_poll_status(const int32_t *status_dev, void *stream);

/* ---- user side ---------------------------------------------------------- */

/*
 * Error correction + fp conversion + memory update (Algorithm 1, the user's conversion
 * step and memory-update step), for all users:
 *     x = fl32(g + fl32(gamma * err));  sym = Q_A(x);  err = fl32(x - value_A(sym))
 * Q_A rounds to the nearest level, ties to the even multiple of the local quantum;
 * magnitudes above the top level saturate to it (the excess stays in err).
 *
 *   g      [U][stride] f32 in     gradients
 *   err    [U][stride] f32 in/out memory m_{t-1} -> m_t (the only in/out buffer)
 *   sym    [U][stride] u8  out    symbols
 *   seg_off [nseg+1] i64 in       segment (tensor) boundaries, seg_off[0] = 0,
 *                                 non-decreasing, seg_off[nseg] = n; NULL = one segment
 *   anchor [U][nseg] i32          per anchor_mode; with FROM_ABSMAX_G it is computed as
 *                                 floor(log2 max|g|) over the segment, clamped to
 *                                 [2^E - 127, 127], from g (not from g + gamma*err)
 *   counts [U][K] u32 out         optional (NULL to skip): symbol histogram of each user,
 *                                 overwritten -- the fused form of co3_histogram
 * n = 0 is allowed.  Non-finite inputs are not rejected: Inf saturates, NaN is unspecified.
 */
int32_t co3_convert_ef(const float *g, float *err, uint8_t *sym, int64_t n, int32_t U, int64_t stride,
                       const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode, float gamma,
                       co3_fmt fmt, uint32_t *counts, void *stream);

/*
 * The bias of Sec. III (i) in the form the approximation of Sec. IV-B gives it: a real multiplier c per
 * (user, tensor), c = (0.46 - 2.85 b + 5.37 b^2 - 2.85 b^3 + 0.52 b^4) / alpha with (b, alpha) the shape and
 * scale of the GenNorm law fitted to the corrected gradient x = g + gamma*m, applied as
 *     y = fl32(c * x);  sym = Q_A(y);  ghat = fl32(value_A(sym) / c);  err = fl32(x - ghat)
 * on the fixed grid of the given anchor A (2^(E-1) is the IEEE-style choice; the 4-bit format of the
 * paper is E = 1, M = 2, A = 1).  Three calls:
 *
 * co3_moments: sums[u][s] = (sum |x|, sum x^2) over tensor s of user u, accumulated in fp64 (the order of
 *   the additions is unspecified: results agree with a sequential sum to about 1e-13 relative).
 *     sums [U][nseg][2] f64 out, overwritten; g, err, seg_off, nseg, gamma as in co3_convert_ef
 * co3_bias_scale: moment matching, (sum|x|)^2 / (count * sum x^2) = Gamma(2/b)^2 / (Gamma(1/b) Gamma(3/b))
 *   solved for b in [0.05, 50], alpha from the second moment; b limited to [0.4, 1.6] (the range the paper
 *   plots) inside the polynomial; c kept within [2^-96, 2^96]; a tensor of zeros gets c = 1.
 *     scale [U][nseg] f32 out;  fit [U][nseg][2] f64 out, optional (NULL to skip): (b, alpha) before limiting
 * co3_convert_ef_scaled: co3_convert_ef with anchor given (input) and the multipliers scale [U][nseg].
 */
int32_t co3_moments(const float *g, const float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                    int32_t nseg, float gamma, double *sums, void *stream);
int32_t co3_bias_scale(const double *sums, int64_t n, int32_t U, const int64_t *seg_off, int32_t nseg, float *scale,
                       double *fit, void *stream);
int32_t co3_convert_ef_scaled(const float *g, float *err, uint8_t *sym, int64_t n, int32_t U, int64_t stride,
                              const int64_t *seg_off, int32_t nseg, const int32_t *anchor, const float *scale,
                              float gamma, co3_fmt fmt, uint32_t *counts, void *stream);

/*
 * Empirical symbol counts per user (the stand-in for the symbol law that the Huffman
 * design of Sec. III (ii) needs): counts[u][k] = #{i < n : sym[u][i] = k}, overwritten.
 * Symbols >= K (cannot come from co3_convert_ef) are ignored.  n < 2^32.
 */
int32_t co3_histogram(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, uint32_t *counts,
                      void *stream);

/*
 * Huffman code per user from integer weights (Sec. III (ii)): empirical counts, or model
 * weights of a quantised GenNorm law (co3_model_weights).  Symbols with weight 0 get no code.
 * Lengths follow the two-queue construction on leaves sorted by (weight, symbol), a leaf
 * winning a weight tie against a merged node; one active symbol gets the 1-bit code "0".
 * Codewords are canonical: ordered by (length, symbol), first all zeros, each next one
 * (previous + 1) << (length growth).
 *
 *   weights [U][K] u32 in
 *   codes   [U][CO3_CODE_BYTES] out; bytes 0..K-1 of each blob are len[K]; the rest
 *           (codewords, decoder tables) is private to the library.
 */
int32_t co3_build_code(const uint32_t *weights, int32_t U, co3_fmt fmt, void *codes, int32_t *status, void *stream);

/*
 * Compression h_Hf (Algorithm 1, the user's compression step) of every user's symbols with its code.
 *
 *   words        [U][cap_words] u64 out  streams; words past ceil(total_bits/64) are untouched
 *   chunk_syms   64, 128, ..., 4096 (power of two)
 *   chunk_bitoff [U][nchunks+1] u64 out
 *   total_bits   [U] u64 out
 *   workspace    co3_encode_workspace_bytes(n, U) bytes, 8-byte aligned, contents unspecified
 * Device-reported: CO3_ENOCODE; CO3_ECAP (nothing is written past cap_words, total_bits still
 * reports the needed length, the words of that user are unspecified).
 */
int32_t co3_encode(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                   uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                   uint64_t *total_bits, void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/*
 * co3_encode for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture that owns no buffers, tight serving loops, harnesses that forbid allocation): same arguments,
 * same results bit for bit, the tile and group sizes living in a fixed array of
 * CO3_ENCODE_STATIC_WS_BYTES bytes inside the library's device image (one copy per GPU, held until the
 * process ends).  The call allocates and frees nothing.  Batches with
 * co3_encode_workspace_bytes(n, U) > CO3_ENCODE_STATIC_WS_BYTES are rejected with CO3_EINVAL (the limit
 * admits about 5 * 10^8 symbols over all users).  All calls on one GPU share the array: calls that
 * overlap on one GPU (two streams, two threads) race and must be serialised by the caller; nothing in
 * the array needs to start at zero, every entry that is read was written by the same call.
 */
#define CO3_ENCODE_STATIC_WS_BYTES (4u << 20)
int32_t co3_encode_static(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                          uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                          uint64_t *total_bits, int32_t *status, void *stream);

/* ---- parameter-server side ---------------------------------------------- */

/*
 * Decompression (Algorithm 1, the parameter server's decompression step): the inverse of
 * co3_encode, chunk by chunk.  sym_out [U][stride] u8.  Device-reported: CO3_EBADSTREAM.
 */
int32_t co3_decode(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                   const void *codes, co3_fmt fmt, int64_t n, int32_t U, uint8_t *sym_out, int64_t stride,
                   int32_t *status, void *stream);

/*
 * Decompression + average over users (Sec. II-A, the aggregate (1/U) * sum_u ghat^(u); the
 * learning-rate step on the model is the caller's):
 *     avg[i] = fl32( (((0 + v_0) + v_1) + ... + v_{U-1}) / U ),  v_u = value_{A_u}(symbol i of user u)
 * added in user-index order in fp32, one fp32 division.
 *
 *   anchor    [U][nseg] i32 in, seg_off as in co3_convert_ef
 *   avg_out   [n] f32 out
 *   workspace co3_ps_aggregate_workspace_bytes(n, U, chunk_syms) bytes, 16-byte aligned; holds the
 *             decoded symbols in a private interleaved order
 */
int32_t co3_ps_aggregate(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                         const void *codes, co3_fmt fmt, int64_t n, int32_t U, const int32_t *anchor,
                         const int64_t *seg_off, int32_t nseg, float *avg_out, void *workspace, size_t ws_bytes,
                         int32_t *status, void *stream);

/*
 * The aggregate of Sec. II-A taken over the users in groups: co3_ps_aggregate that continues a sum and
 * may leave it undivided,
 *     out[i] = fl32( ((acc_in[i] + v_0) + v_1) + ... + v_{U-1} ) [ / divide_by ]
 * with acc_in = NULL read as zeros and no division when divide_by = 0.  Calling it for the users
 * 0..a-1 (acc_in NULL, divide_by 0), then a..b-1 with the first result as acc_in, ..., the last group with
 * divide_by = the number of all users, performs the additions and the one division of co3_ps_aggregate
 * over all users in the same order: the result is the same bit for bit.  The groups' decoders can then
 * run as soon as a group's streams are there.
 *   acc_in    [n] f32 in or NULL; may be the same array as out
 *   out       [n] f32 out
 *   other arguments, workspace and errors as co3_ps_aggregate (U = users of this group, pointers at the
 *   group's first user); CO3_EINVAL when divide_by < 0
 */
int32_t co3_ps_aggregate_partial(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                 int32_t chunk_syms, const void *codes, co3_fmt fmt, int64_t n, int32_t U,
                                 const int32_t *anchor, const int64_t *seg_off, int32_t nseg, const float *acc_in,
                                 int32_t divide_by, float *out, void *workspace, size_t ws_bytes, int32_t *status,
                                 void *stream);

/*
 * The two halves of co3_ps_aggregate (Alg. 1, PS decompression step; Sec. II-A aggregate) as calls of their
 * own, for a server that decompresses the users' streams in groups -- as they arrive, or on several HIP
 * streams at once -- and averages when all are there:
 *   co3_ps_decode_users  decompresses the streams of U consecutive users (pointers at the first of them) into
 *                        their places first_user .. first_user + U - 1 of the averaging workspace of U_total
 *                        users (co3_ps_aggregate_workspace_bytes(n, U_total, chunk_syms) bytes)
 *   co3_ps_average       the average of all U users from a workspace that every user has been decompressed
 *                        into: exactly co3_ps_aggregate's second half (same additions, same order)
 * Arguments and errors as co3_ps_aggregate.
 */
int32_t co3_ps_decode_users(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                            const void *codes, co3_fmt fmt, int64_t n, int32_t U, int32_t first_user, int32_t U_total,
                            void *workspace, size_t ws_bytes, int32_t *status, void *stream);
int32_t co3_ps_average(const void *workspace, size_t ws_bytes, int32_t chunk_syms, co3_fmt fmt, int64_t n, int32_t U,
                       const int32_t *anchor, const int64_t *seg_off, int32_t nseg, float *avg_out, void *stream);

/*
 * co3_ps_aggregate for streams made with co3_convert_ef_scaled: v_u = fl32(value_{A_u}(symbol) / c_u) with
 * the multipliers scale [U][nseg] of the users (Sec. III (i): the receiver undoes the bias).
 */
int32_t co3_ps_aggregate_scaled(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                int32_t chunk_syms, const void *codes, co3_fmt fmt, int64_t n, int32_t U,
                                const int32_t *anchor, const float *scale, const int64_t *seg_off, int32_t nseg,
                                float *avg_out, void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* ---- one code per layer, shared by all users ---------------------------------- */

/*
 * Sec. III (ii) assigns the codes per layer: every layer has a code of its own, and all users share the
 * code of a layer.  codes is [nseg][CO3_CODE_BYTES], code s serving the
 * elements seg_off[s] .. seg_off[s+1] of every user; build the nseg codes with one call
 * co3_build_code(weights [nseg][K], nseg, ...), the weights being model weights (co3_model_weights) or
 * pooled counts.  The stream of a user is still one concatenation over all its elements, with the same
 * word layout and the same chunk index as co3_encode; only the table that gives element i its codeword
 * changes at the boundaries.  seg_off (device, [nseg+1]) is required.  The boundaries of the codes need
 * not be those of the anchors: a tensor of a few hundred elements cannot pay for a table of its own and
 * is better grouped with a neighbour (the decoder also keeps only four tables resident per workgroup,
 * so runs of tiny groups slow it down); co3_ps_aggregate_layers takes both sets of boundaries.
 *
 * co3_histogram_layers: counts[u][s][k] = #{i in tensor s : sym[u][i] = k}; counts [U][nseg][K] u32 out,
 *   overwritten.  With pool_users != 0 the users are added up: counts [nseg][K], the statistics of the
 *   shared codes (n * U < 2^32).
 * co3_encode_layers / co3_decode_layers: as co3_encode / co3_decode.
 * co3_ps_aggregate_layers: as co3_ps_aggregate, with code_seg_off [code_nseg+1] the boundaries of the codes
 *   and seg_off [nseg+1] those of the anchors; scale may be NULL (no multipliers) or [U][nseg] as in
 *   co3_ps_aggregate_scaled.
 */
int32_t co3_histogram_layers(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                             int32_t nseg, co3_fmt fmt, int32_t pool_users, uint32_t *counts, void *stream);
int32_t co3_encode_layers(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                          const int64_t *seg_off, int32_t nseg, uint64_t *words, int64_t cap_words,
                          int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits, void *workspace,
                          size_t ws_bytes, int32_t *status, void *stream);
int32_t co3_decode_layers(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                          const void *codes, const int64_t *seg_off, int32_t nseg, co3_fmt fmt, int64_t n, int32_t U,
                          uint8_t *sym_out, int64_t stride, int32_t *status, void *stream);
int32_t co3_ps_aggregate_layers(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                int32_t chunk_syms, const void *codes, const int64_t *code_seg_off, int32_t code_nseg,
                                co3_fmt fmt, int64_t n, int32_t U, const int32_t *anchor, const float *scale,
                                const int64_t *seg_off, int32_t nseg, float *avg_out, void *workspace, size_t ws_bytes,
                                int32_t *status, void *stream);

/* ---- fixed codes: conversion and compression in one pass ------------------- */

/*
 * Sec. III (ii) designs the code from a model of the gradients, before the gradients are seen.  With
 * such a code (or one kept from an earlier iteration) the user's three steps of Algorithm 1 need no
 * pass over the symbols of their own: co3_convert_encode gives the results of co3_convert_ef
 * followed by co3_encode with codes[u] -- err, anchor, words, chunk_bitoff, total_bits, bit for
 * bit -- without producing the symbol array or the counts.
 *
 *   arguments  as in co3_convert_ef (g, err, n, U, stride, seg_off, nseg, anchor, anchor_mode, gamma,
 *              fmt) and co3_encode (codes [U], words, cap_words, chunk_syms, chunk_bitoff,
 *              total_bits, status)
 *   workspace  co3_convert_encode_workspace_bytes(n, U, chunk_syms) bytes, 16-byte aligned, contents
 *              unspecified: every 1024 elements pack into a slot of 8 KiB of their own (room for 1024
 *              codewords of any length) before they are moved into the stream, 8 bytes per element
 *              of address space of which a codeword's worth is touched
 *   counts     NULL, or [U][K] u32 out, overwritten: 1 + the number of occurrences of every symbol in this
 *              call.  A code built from them (co3_build_code) has a codeword for every symbol, so it can
 *              serve the next iteration: empirical codes that follow the gradients one iteration behind,
 *              at the cost of one pass (Sec. III (ii) leaves the model of the distribution open)
 *   errors     as the two calls: CO3_EINVAL on the host; CO3_ENOCODE, CO3_ECAP through status (after
 *              CO3_ENOCODE the stream is unspecified)
 *
 * co3_convert_encode_layers is the same pass for one code per layer shared by all users (codes
 * [code_nseg], code_seg_off [code_nseg+1] device, as in co3_encode_layers; the boundaries of the codes
 * need not be those of the anchors), with or without the multipliers of the bias rule: scale NULL gives
 * co3_convert_ef followed by co3_encode_layers; scale [U][nseg] gives co3_convert_ef_scaled followed by
 * co3_encode_layers, and then the anchors are inputs (anchor_mode must be CO3_ANCHOR_GIVEN).  Model
 * codes per layer, the multiplier and one pass together are the scheme of Sec. III as the paper states it.
 * counts: NULL, or [code_nseg][K] u32 out, overwritten: 1 + the occurrences of every symbol in the
 * elements of a code, added up over the users (n * U < 2^32): the weights of the next iteration's codes.
 */
size_t co3_convert_encode_workspace_bytes(int64_t n, int32_t U, int32_t chunk_syms);
int32_t co3_convert_encode(const float *g, float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                           int32_t nseg, int32_t *anchor, int32_t anchor_mode, float gamma, co3_fmt fmt, const void *codes,
                           uint32_t *counts, uint64_t *words, int64_t cap_words, int32_t chunk_syms,
                           uint64_t *chunk_bitoff, uint64_t *total_bits, void *workspace, size_t ws_bytes, int32_t *status,
                           void *stream);
int32_t co3_convert_encode_layers(const float *g, float *err, int64_t n, int32_t U, int64_t stride,
                                  const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode,
                                  const float *scale, float gamma, co3_fmt fmt, const void *codes,
                                  const int64_t *code_seg_off, int32_t code_nseg, uint32_t *counts, uint64_t *words,
                                  int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits,
                                  void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* ---- the user's steps of Algorithm 1 in one call ------------------------------ */

/*
 * Conversion with error correction, memory update, symbol statistics, Huffman code and compression
 * (Algorithm 1, every step of a user between the local gradient and the uplink; Sec. III (i)-(iii)) for
 * all users, with the anchor from max|g| and one empirical code per user: the results of
 *     co3_convert_ef(..., CO3_ANCHOR_FROM_ABSMAX_G, ..., counts) -> co3_build_code(counts) -> co3_encode
 * bit for bit -- err, anchor, counts, codes, words, chunk_bitoff, total_bits (and sym, if asked for).
 * What the one call adds is that it may keep data on the chip between the steps: where a user's
 * gradient fits the register files of the device (with one anchor per user, nseg = 1, for the larger
 * vectors with a part of it in LDS: n up to 98,304 elements per compute unit, 25.1 M on 256 units;
 * with several tensors per user up to 65,536 elements per compute unit, 511 tensors and six users),
 * a single resident grid reads every gradient once, taking the largest magnitudes and converting from
 * the chip, the workgroups exchanging their maxima through words in the workspace; other batches run
 * the separate kernels of the three calls.
 *
 *   arguments  as in co3_convert_ef (g, err, n, U, stride, seg_off, nseg, anchor [out], gamma, fmt,
 *              counts [out, required]), co3_build_code (codes [out]) and co3_encode (words, cap_words,
 *              chunk_syms, chunk_bitoff, total_bits, status)
 *   sym        [U][stride] u8 out, or NULL when the caller has no use for the symbols (the workspace
 *              then holds them where the path needs them)
 *   workspace  co3_user_encode_workspace_bytes(n, U, stride, nseg, sym != NULL) bytes, 256-byte aligned,
 *              contents unspecified
 *   errors     as the three calls; CO3_ETIMEOUT through status when a wait of the resident grid ran
 *              out (every such wait is bounded, see co3_set_exchange_spin_limit); the outputs are
 *              then unspecified
 * The resident grid assumes that its workgroups (one per compute unit at most) can all be on the device
 * at once.  Kernels of other streams that share the device only delay that; they cannot prevent it --
 * except another resident grid: two of them started at the same time may each hold part of the device and
 * wait for the rest, until both time out.  Calls that may run at the same time (on different streams) must
 * not both take the resident-grid path.
 */
size_t co3_user_encode_workspace_bytes(int64_t n, int32_t U, int64_t stride, int32_t nseg, int32_t caller_has_sym);
int32_t co3_user_encode(const float *g, float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                        int32_t nseg, int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, void *codes,
                        uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                        uint64_t *total_bits, uint8_t *sym, void *workspace, size_t ws_bytes, int32_t *status,
                        void *stream);

/*
 * Bound on the number of polls of one wait inside the resident grid of co3_user_encode (process-wide;
 * default 2^18, each poll takes on the order of a microsecond; a negative value restores the default).
 * A wait that runs out raises CO3_ETIMEOUT and the kernel goes on to its end.  With 0 no wait ever
 * polls, so every wait runs out at once: how a test forces that path from the host.
 */
void co3_set_exchange_spin_limit(int64_t polls);

/* ---- launch timing (diagnostic) ------------------------------------------ */

/*
 * Optional per-kernel timing with HIP events recorded on the launch stream, for benchmarks
 * that must report one kernel's average duration.  Process-global and not thread-safe: the
 * only state the library keeps, and only while enabled.  kernel ids: 0 k_fill_i32, 1 k_absmax,
 * 2 k_convert_ef, 3 k_histogram, 4 k_build_code, 5 k_enc_sizes, 6 k_enc_scan, 7 k_enc_pack,
 * 8 k_decode, 9 k_ps_sum, 10 k_moments, 11 k_bias_scale, 12 k_coop_convert (co3_kernel_name returns
 * these names, "" for other ids).
 *   co3_timing_enable(mask): bracket every later launch of kernel k with events iff bit k is set.
 *   co3_timing_read(k, &ms, &count): waits for the recorded events, then returns the summed
 *       duration and launch count of kernel k since the last reset.
 *   co3_timing_reset(): waits likewise and clears all sums.
 */
#define CO3_KERNEL_COUNT 13
int32_t co3_timing_enable(uint32_t kernel_mask);
int32_t co3_timing_read(int32_t kernel, double *total_ms, int64_t *launches);
int32_t co3_timing_reset(void);
const char *co3_kernel_name(int32_t kernel);

/* ---- model table (host only) -------------------------------------------- */

/*
 * Integer Huffman weights of a GenNorm(beta, scale alpha) source quantised with anchor A
 * (Sec. III (ii): the code is designed from the assumed GenNorm law, not from data).
 * Cell boundaries are the midpoints between adjacent levels, the zero cell is symmetric, the
 * top cell is unbounded; weight = round(p * 2^32) kept within [1, 2^32-1]; the negative-zero
 * symbol gets 0.  weights_host: HOST pointer to K uint32.  Pure host arithmetic.
 */
int32_t co3_model_weights(int32_t A, co3_fmt fmt, double beta, double alpha, uint32_t *weights_host);

/*
 * Model tables of codes shared by the users, one per group of consecutive tensors (Sec. III (ii): the
 * codes are assigned per layer and designed from the GenNorm law of the layer; Sec. IV-B: that law is
 * fitted per tensor).  The law of group k is the one fitted to the group's largest tensor among those
 * that start inside the group (the first of equals; the tensor that holds the group's first element when
 * none starts there), pooled over the users:
 *     beta  = (sum over u of fit[u][s][0]) / U,   alpha = (sum over u of fit[u][s][1] * scale[u][s]) / U
 * -- shape and scale of what is rounded onto the grid, the multiplied corrected gradient -- added in
 * user order in double precision; beta is kept within [0.2, 4], alpha at or above 1e-30; the weights are
 * co3_model_weights(A, fmt, beta, alpha).
 *   fit           [U][nseg][2] f64 (shape, scale) as co3_bias_scale returns them;  scale [U][nseg] f32
 *   seg_off       [nseg + 1] tensor boundaries;  code_seg_off [ncodes + 1] group boundaries
 *   weights_host  [ncodes][K] u32 out
 * All pointers are HOST pointers; pure host arithmetic.  CO3_EINVAL on bad arguments.
 */
int32_t co3_design_layer_tables(const double *fit, const float *scale, int32_t U, int32_t nseg, const int64_t *seg_off,
                                const int64_t *code_seg_off, int32_t ncodes, int32_t A, co3_fmt fmt,
                                uint32_t *weights_host);

#ifdef __cplusplus
}
#endif
#endif /* CO3_H */
