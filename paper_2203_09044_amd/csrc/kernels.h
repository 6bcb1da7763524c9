// Host-side launchers of the libco3 kernels (one per kernel; arguments already validated).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/co3.h"

// Kernel ids for the optional launch timing (co3_timing_* in the public header).
enum Co3Kernel {
    CO3_K_FILL = 0, CO3_K_ABSMAX, CO3_K_CONVERT, CO3_K_HISTOGRAM, CO3_K_BUILD, CO3_K_ENC_SIZES, CO3_K_ENC_SCAN,
    CO3_K_ENC_PACK, CO3_K_DECODE, CO3_K_PS_SUM, CO3_K_MOMENTS, CO3_K_BIAS_SCALE, CO3_K_COOP, CO3_K_COUNT
};

// Brackets one kernel launch with a pair of HIP events on the launch stream when timing of that
// kernel is enabled; otherwise does nothing.
struct Co3LaunchTimer {
    Co3LaunchTimer(int kernel, hipStream_t st);
    ~Co3LaunchTimer();
    int slot;
    hipStream_t stream;
};

hipError_t co3_launch_fill(int32_t *a, int64_t na, int32_t va, uint32_t *b, int64_t nb, hipStream_t st, uint32_t vb = 0u);
hipError_t co3_launch_absmax(const float *g, int64_t n, int U, int64_t stride, const int64_t *seg_off, int nseg,
                             int32_t *anchor, hipStream_t st);
hipError_t co3_launch_convert(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride,
                              const int64_t *seg_off, int nseg, const int32_t *anchor, const float *scale, float gamma,
                              co3_fmt fmt, uint32_t *counts, hipStream_t st, int sym_nib = 0);
// sym_nib (alphabets of at most 16 symbols, counts given, no multiplier): the symbols leave two per byte, the
// earlier one in the low half, rows of stride / 2 bytes -- the form the encoder reads with its own sym_nib
// resident-grid conversion (anchor from max|g| and conversion with one read of g; one anchor per user);
// slots: [U][grid] u32 exchange words, counts_rep: [CO3_COOP_COUNT_REPS][U][K] partial counts, both zero at launch
// nseg > 1 (seg_off given): one anchor per (user, tensor), anchor [U][nseg], tmax: U * nseg zero words
bool co3_coop_fits(int64_t n, int nseg, int cus, int *kpt_out, int *grid_out);
hipError_t co3_launch_coop_convert(const float *g, float *err, uint8_t *sym, int64_t n, int U, int64_t stride, int kpt,
                                   int grid, const int64_t *seg_off, int nseg, int32_t *anchor, float gamma, co3_fmt fmt,
                                   uint32_t *counts_rep, uint32_t *slots, uint32_t *tmax, uint32_t spin_limit,
                                   int32_t *status, int sym_nib, hipStream_t st);
hipError_t co3_launch_histogram(const uint8_t *sym, int64_t n, int U, int64_t stride, int K, uint32_t *counts,
                                hipStream_t st);
// nrep > 1: weights is [nrep][U][K] partial tables that the kernel adds up (the sums also go to sums_out [U][K])
hipError_t co3_launch_build_code(const uint32_t *weights, int U, int K, void *codes, int32_t *status, hipStream_t st,
                                 int nrep = 1, uint32_t *sums_out = nullptr);
// After a resident-grid conversion that left the ragged end [n_full, n) of every user unconverted: that end,
// the user's counts (its own + the nrep partial tables [nrep][U][K]) and the user's code; all pointers at user 0
// of the batch of U, the launch serving users first_user .. first_user + users - 1
hipError_t co3_launch_user_finish(const float *g, float *err, uint8_t *sym, int64_t n, int64_t n_full, int64_t stride, int U,
                                  const int64_t *seg_off, int nseg, const int32_t *anchor, float gamma, co3_fmt fmt,
                                  int sym_nib, const uint32_t *counts_rep, int nrep, uint32_t *counts, void *codes,
                                  int32_t *status, hipStream_t st, int first_user, int users);
// elements of a user that the resident grid converts itself (a whole number of wavefront parts)
int64_t co3_coop_full_elements(int64_t n, int kpt);
#define CO3_COOP_COUNT_REPS 32   // partial count tables of the resident-grid user side (workgroup w adds to table w mod 32)
hipError_t co3_launch_encode(const uint8_t *sym, int64_t n, int U, int64_t stride, const void *codes, int K,
                             const int64_t *seg_off, int nseg, uint64_t *words, int64_t cap_words, int chunk_syms,
                             uint64_t *chunk_bitoff, uint64_t *total_bits, uint64_t *tilesum, int32_t *status,
                             hipStream_t st, int sym_nib = 0);
// device address, on the current device, of the library's own fixed encoder workspace of
// CO3_ENCODE_STATIC_WS_BYTES bytes (looked up on the first call per device; allocates nothing)
hipError_t co3_static_encode_workspace(void **ptr_out);
// the scan pass of the encoder alone: sizes[U][nsizes] -> exclusive offsets in place, stream length, capacity check
hipError_t co3_launch_enc_scan(uint64_t *sizes, int64_t nsizes, int U, int64_t cap_words, uint64_t *chunk_bitoff,
                               int64_t nchunks, uint64_t *total_bits, int32_t *status, hipStream_t st);
size_t co3_fused_workspace_bytes_impl(int64_t n, int U, int chunk_syms);
hipError_t co3_launch_convert_encode(const float *g, float *err, int64_t n, int U, int64_t stride, const int64_t *seg_off,
                                     int nseg, const int32_t *anchor, const float *scale, float gamma, co3_fmt fmt,
                                     const void *codes, const int64_t *code_seg_off, int ncodes, uint32_t *counts,
                                     uint64_t *words, int64_t cap_words, int chunk_syms, uint64_t *chunk_bitoff,
                                     uint64_t *total_bits, void *workspace, int32_t *status, hipStream_t st);
hipError_t co3_launch_decode(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int chunk_syms,
                             const void *codes, const int64_t *seg_off, int nseg, int K, int64_t n, int U,
                             uint8_t *sym_out, int64_t stride, int tiled, int32_t *status, hipStream_t st);
// The averaging workspace holds two symbols per byte when this is true: alphabets of at most 16 symbols,
// chunks of at least two runs of 32, and one code per user or one code shared by everything
// (code_groups = 0 for per-user codes, else the number of shared per-layer codes).  The decoder then
// also reads two symbols per lookup.
static inline bool co3_ws_packed(int K, int chunk_syms, int code_groups)
{
    return code_groups <= 1 && K <= 16 && chunk_syms >= 64;
}
// out[i] = (acc_in ? acc_in[i] : 0) + sum over the U users in order, divided by `divisor` when it is positive
hipError_t co3_launch_ps_sum_tiled(const uint8_t *symt, int64_t n, int U, int64_t ws_stride, int chunk_syms,
                                   const int32_t *anchor, const float *scale, const int64_t *seg_off, int nseg,
                                   co3_fmt fmt, int packed, const float *acc_in, float divisor, float *avg_out,
                                   hipStream_t st);
hipError_t co3_launch_moments(const float *g, const float *err, int64_t n, int U, int64_t stride,
                              const int64_t *seg_off, int nseg, float gamma, double *sums, hipStream_t st);
hipError_t co3_launch_bias_scale(const double *sums, int64_t n, int U, const int64_t *seg_off, int nseg, float *scale,
                                 double *fit, hipStream_t st);
hipError_t co3_launch_histogram_layers(const uint8_t *sym, int64_t n, int U, int64_t stride, int K,
                                       const int64_t *seg_off, int nseg, int pool_users, uint32_t *counts,
                                       hipStream_t st);
