// extern "C" boundary of libco3: argument validation and kernel sequencing only.
#include <math.h>

#include "co3_dev.h"
#include "kernels.h"

#include <atomic>
#include <vector>

namespace {

// ---- compute units of each device, looked up once -------------------------------------------
int device_cus()
{
    static std::atomic<int> cus_of[64];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int c = cus_of[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || c < 1) return 0;
        cus_of[dev].store(c, std::memory_order_relaxed);
    }
    return c;
}

std::atomic<uint32_t> g_spin_limit{1u << 18};

size_t round_up_256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- optional launch timing (diagnostic, process-global, not thread-safe) ------------------
struct TimedLaunch {
    hipEvent_t start, stop;
    int kernel;
    bool pending;
};
uint32_t g_timing_mask = 0;
std::vector<TimedLaunch> g_timed;                 // event pairs, reused after each read
size_t g_timed_used = 0;
double g_total_ms[CO3_K_COUNT] = {0};
int64_t g_launches[CO3_K_COUNT] = {0};

int timing_acquire(int kernel)
{
    if (g_timed_used == g_timed.size()) {
        TimedLaunch t{};
        if (hipEventCreate(&t.start) != hipSuccess) return -1;
        if (hipEventCreate(&t.stop) != hipSuccess) return -1;
        g_timed.push_back(t);
    }
    g_timed[g_timed_used].kernel = kernel;
    g_timed[g_timed_used].pending = true;
    return (int)g_timed_used++;
}

void timing_collect()
{
    for (size_t i = 0; i < g_timed_used; ++i) {
        TimedLaunch &t = g_timed[i];
        if (!t.pending) continue;
        float ms = 0.f;
        if (hipEventSynchronize(t.stop) == hipSuccess && hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) {
            g_total_ms[t.kernel] += ms;
            g_launches[t.kernel] += 1;
        }
        t.pending = false;
    }
    g_timed_used = 0;
}

bool fmt_ok(co3_fmt f)
{
    return f.exp_bits >= 1 && f.mant_bits >= 0 && 1 + f.exp_bits + f.mant_bits <= 8;
}

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

bool batch_ok(int64_t n, int32_t U, int64_t stride)
{
    if (n < 0 || U < 1 || n >= ((int64_t)1 << 32)) return false;
    if (U > 1 && (stride < n || stride % 16 != 0)) return false;
    return true;
}

bool chunk_ok(int32_t c) { return c >= 64 && c <= 4096 && (c & (c - 1)) == 0; }

int32_t hip_rc(hipError_t e) { return e == hipSuccess ? CO3_OK : CO3_EHIP; }

}  // namespace

Co3LaunchTimer::Co3LaunchTimer(int kernel, hipStream_t st) : slot(-1), stream(st)
{
    if (g_timing_mask & (1u << kernel)) {
        slot = timing_acquire(kernel);
        if (slot >= 0) (void)hipEventRecord(g_timed[slot].start, stream);
    }
}

Co3LaunchTimer::~Co3LaunchTimer()
{
    if (slot >= 0) (void)hipEventRecord(g_timed[slot].stop, stream);
}

extern "C" {

int32_t co3_timing_enable(uint32_t kernel_mask)
{
    g_timing_mask = kernel_mask & ((1u << CO3_K_COUNT) - 1u);
    return CO3_OK;
}

int32_t co3_timing_read(int32_t kernel, double *total_ms, int64_t *launches)
{
    if (kernel < 0 || kernel >= CO3_K_COUNT || !total_ms || !launches) return CO3_EINVAL;
    timing_collect();
    *total_ms = g_total_ms[kernel];
    *launches = g_launches[kernel];
    return CO3_OK;
}

int32_t co3_timing_reset(void)
{
    timing_collect();
    for (int k = 0; k < CO3_K_COUNT; ++k) {
        g_total_ms[k] = 0;
        g_launches[k] = 0;
    }
    return CO3_OK;
}

const char *co3_kernel_name(int32_t kernel)
{
    static const char *names[CO3_K_COUNT] = {"k_fill_i32", "k_absmax",    "k_convert_ef", "k_histogram", "k_build_code",
                                             "k_enc_sizes", "k_enc_scan", "k_enc_pack",   "k_decode",    "k_ps_sum",
                                             "k_moments",  "k_bias_scale", "k_coop_convert"};
    return (kernel >= 0 && kernel < CO3_K_COUNT) ? names[kernel] : "";
}

const char *co3_strerror(int32_t status)
{
    switch (status) {
    case CO3_OK: return "ok";
    case CO3_EINVAL: return "invalid argument";
    case CO3_ECAP: return "stream capacity exceeded";
    case CO3_ENOCODE: return "symbol without a codeword";
    case CO3_EBADSTREAM: return "inconsistent stream";
    case CO3_EHIP: return "HIP runtime error";
    case CO3_ETIMEOUT: return "bounded wait inside a kernel ran out";
    default: return "unknown status";
    }
}

size_t co3_encode_workspace_bytes(int64_t n, int32_t U)
{
    if (n < 0 || U < 1) return 0;
    int64_t nblk = (n + CO3_PACK_SYMS - 1) / CO3_PACK_SYMS;
    int64_t ngrp = (nblk + CO3_PACK_GROUP - 1) / CO3_PACK_GROUP;
    return (size_t)((nblk > 0 ? nblk : 1) + (ngrp > 0 ? ngrp : 1)) * (size_t)U * sizeof(uint64_t);
}

size_t co3_convert_encode_workspace_bytes(int64_t n, int32_t U, int32_t chunk_syms)
{
    if (n < 0 || U < 1 || !chunk_ok(chunk_syms)) return 0;
    return co3_fused_workspace_bytes_impl(n, U, chunk_syms);
}

size_t co3_ps_aggregate_workspace_bytes(int64_t n, int32_t U, int32_t chunk_syms)
{
    if (n < 0 || U < 1 || !chunk_ok(chunk_syms)) return 0;
    int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;
    int64_t ntiles = (nchunks + CO3_WAVE - 1) / CO3_WAVE;
    if (ntiles < 1) ntiles = 1;
    return (size_t)ntiles * CO3_WAVE * (size_t)chunk_syms * (size_t)U;
}

int64_t co3_cap_words_empirical(int64_t n, co3_fmt fmt)
{
    if (n < 0 || !fmt_ok(fmt)) return 0;
    int64_t w = (n * (1 + fmt.exp_bits + fmt.mant_bits) + 63) / 64;
    return (w + 1) & ~(int64_t)1;
}

int32_t co3_poll_status(const int32_t *status_dev, void *stream)
{
    if (!status_dev) return CO3_EINVAL;
    int32_t h = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&h, status_dev, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CO3_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return CO3_EHIP;
    return h;
}

static int32_t convert_common(const float *g, float *err, uint8_t *sym, int64_t n, int32_t U, int64_t stride,
                              const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode,
                              const float *scale, float gamma, co3_fmt fmt, uint32_t *counts, void *stream, int sym_nib = 0)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || nseg < 1 || (seg_off == nullptr && nseg != 1)) return CO3_EINVAL;
    if (!g || !err || !sym || !anchor) return CO3_EINVAL;
    if (!aligned(g, 16) || !aligned(err, 16) || !aligned(sym, 16)) return CO3_EINVAL;
    if (anchor_mode != CO3_ANCHOR_GIVEN && anchor_mode != CO3_ANCHOR_FROM_ABSMAX_G) return CO3_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FmtC fc(fmt);
    const bool from_g = anchor_mode == CO3_ANCHOR_FROM_ABSMAX_G;
    hipError_t e = co3_launch_fill(from_g ? anchor : nullptr, from_g ? (int64_t)U * nseg : 0, fc.F - 126, counts,
                                   counts ? (int64_t)U * fc.K : 0, st);
    if (e != hipSuccess) return CO3_EHIP;
    if (from_g) {
        e = co3_launch_absmax(g, n, U, stride, seg_off, nseg, anchor, st);
        if (e != hipSuccess) return CO3_EHIP;
    }
    return hip_rc(co3_launch_convert(g, err, sym, n, U, stride, seg_off, nseg, anchor, scale, gamma, fmt, counts, st,
                                     sym_nib));
}

int32_t co3_convert_ef(const float *g, float *err, uint8_t *sym, int64_t n, int32_t U, int64_t stride,
                       const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode, float gamma,
                       co3_fmt fmt, uint32_t *counts, void *stream)
{
    return convert_common(g, err, sym, n, U, stride, seg_off, nseg, anchor, anchor_mode, nullptr, gamma, fmt, counts,
                          stream);
}

int32_t co3_convert_ef_scaled(const float *g, float *err, uint8_t *sym, int64_t n, int32_t U, int64_t stride,
                              const int64_t *seg_off, int32_t nseg, const int32_t *anchor, const float *scale,
                              float gamma, co3_fmt fmt, uint32_t *counts, void *stream)
{
    if (!scale) return CO3_EINVAL;
    return convert_common(g, err, sym, n, U, stride, seg_off, nseg, const_cast<int32_t *>(anchor), CO3_ANCHOR_GIVEN,
                          scale, gamma, fmt, counts, stream);
}

static int32_t convert_encode_common(const float *g, float *err, int64_t n, int32_t U, int64_t stride,
                                     const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode,
                                     const float *scale, float gamma, co3_fmt fmt, const void *codes,
                                     const int64_t *code_seg_off, int32_t ncodes, uint32_t *counts, uint64_t *words,
                                     int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits,
                                     void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || nseg < 1 || (seg_off == nullptr && nseg != 1)) return CO3_EINVAL;
    if (!chunk_ok(chunk_syms) || cap_words < 0 || cap_words % 2 != 0) return CO3_EINVAL;
    if (!g || !err || !anchor || !codes || !words || !chunk_bitoff || !total_bits || !workspace) return CO3_EINVAL;
    if (!aligned(g, 16) || !aligned(err, 16) || !aligned(words, 16) || !aligned(codes, 8) || !aligned(workspace, 16))
        return CO3_EINVAL;
    if (anchor_mode != CO3_ANCHOR_GIVEN && anchor_mode != CO3_ANCHOR_FROM_ABSMAX_G) return CO3_EINVAL;
    if (scale && anchor_mode != CO3_ANCHOR_GIVEN) return CO3_EINVAL;      // the multiplier belongs to a fixed grid
    if (scale && !code_seg_off) return CO3_EINVAL;                        // ... and goes with the per-layer codes
    // counts pooled over the users are 32-bit: every symbol of every user may land in one counter
    if (counts && code_seg_off && (int64_t)n * U >= ((int64_t)1 << 32) - 1) return CO3_EINVAL;
    if (ws_bytes < co3_convert_encode_workspace_bytes(n, U, chunk_syms)) return CO3_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FmtC fc(fmt);
    const bool from_g = anchor_mode == CO3_ANCHOR_FROM_ABSMAX_G;
    if (from_g || counts) {          // anchors start at the lower clamp, the counts at one
        const int64_t ncounts = (int64_t)(code_seg_off ? ncodes : U) * fc.K;      // per code group, else per user
        hipError_t e = co3_launch_fill(from_g ? anchor : nullptr, from_g ? (int64_t)U * nseg : 0, fc.F - 126, counts,
                                       counts ? ncounts : 0, st, 1u);
        if (e != hipSuccess) return CO3_EHIP;
    }
    if (from_g) {
        hipError_t e = co3_launch_absmax(g, n, U, stride, seg_off, nseg, anchor, st);
        if (e != hipSuccess) return CO3_EHIP;
    }
    return hip_rc(co3_launch_convert_encode(g, err, n, U, stride, seg_off, nseg, anchor, scale, gamma, fmt, codes,
                                            code_seg_off, ncodes, counts, words, cap_words, chunk_syms, chunk_bitoff,
                                            total_bits, workspace, status, st));
}

int32_t co3_convert_encode(const float *g, float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                           int32_t nseg, int32_t *anchor, int32_t anchor_mode, float gamma, co3_fmt fmt, const void *codes,
                           uint32_t *counts, uint64_t *words, int64_t cap_words, int32_t chunk_syms,
                           uint64_t *chunk_bitoff, uint64_t *total_bits, void *workspace, size_t ws_bytes, int32_t *status,
                           void *stream)
{
    return convert_encode_common(g, err, n, U, stride, seg_off, nseg, anchor, anchor_mode, nullptr, gamma, fmt, codes,
                                 nullptr, 0, counts, words, cap_words, chunk_syms, chunk_bitoff, total_bits, workspace,
                                 ws_bytes, status, stream);
}

int32_t co3_convert_encode_layers(const float *g, float *err, int64_t n, int32_t U, int64_t stride,
                                  const int64_t *seg_off, int32_t nseg, int32_t *anchor, int32_t anchor_mode,
                                  const float *scale, float gamma, co3_fmt fmt, const void *codes,
                                  const int64_t *code_seg_off, int32_t code_nseg, uint32_t *counts, uint64_t *words,
                                  int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits,
                                  void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!code_seg_off || code_nseg < 1) return CO3_EINVAL;
    return convert_encode_common(g, err, n, U, stride, seg_off, nseg, anchor, anchor_mode, scale, gamma, fmt, codes,
                                 code_seg_off, code_nseg, counts, words, cap_words, chunk_syms, chunk_bitoff, total_bits,
                                 workspace, ws_bytes, status, stream);
}

void co3_set_exchange_spin_limit(int64_t polls)
{
    g_spin_limit.store(polls < 0 ? (1u << 18) : polls > 0xffffffffll ? 0xffffffffu : (uint32_t)polls);
}

// Layout of the workspace of co3_user_encode: the encoder's workspace, the symbols [U][stride] where the
// caller passes no array for them, and, where the resident grid serves the batch, its exchange words
// [U][workgroups] u32 and partial count tables [CO3_COOP_COUNT_REPS][U][K] u32.
// Several tensors per user: the resident grid pays an exchange of the tensors' maxima per user, which the
// separate kernels do not; measured on 62 tensors of 11.2 M elements (us, resident | separate): one user
// 48 | 68, four 164 | 157, ten 392 | 380: 48 + 38 per further user against 68 + 35, so it is taken up to six.
#ifndef CO3_COOP_SEGS_MAX_USERS
#define CO3_COOP_SEGS_MAX_USERS 6
#endif
static bool user_encode_coop(int64_t n, int32_t U, int32_t nseg, int *kpt, int *grid)
{
    const int cus = device_cus();
    if (nseg > 1 && U > CO3_COOP_SEGS_MAX_USERS) return false;
    return cus > 0 && co3_coop_fits(n, nseg, cus, kpt, grid);
}

size_t co3_user_encode_workspace_bytes(int64_t n, int32_t U, int64_t stride, int32_t nseg, int32_t caller_has_sym)
{
    if (n < 0 || U < 1 || stride < 0 || nseg < 1) return 0;
    size_t b = round_up_256(co3_encode_workspace_bytes(n, U));
    if (!caller_has_sym) b += round_up_256((size_t)U * (size_t)(stride > n ? stride : n) + 16);
    int kpt = 0, grid = 0;
    if (user_encode_coop(n, U, nseg, &kpt, &grid)) {
        b += round_up_256((size_t)U * ((size_t)grid + (nseg > 1 ? (size_t)nseg : 0)) * sizeof(uint32_t));
        b += round_up_256((size_t)CO3_COOP_COUNT_REPS * (size_t)U * 256 * sizeof(uint32_t));
    }
    return b;
}

int32_t co3_user_encode(const float *g, float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                        int32_t nseg, int32_t *anchor, float gamma, co3_fmt fmt, uint32_t *counts, void *codes,
                        uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                        uint64_t *total_bits, uint8_t *sym, void *workspace, size_t ws_bytes, int32_t *status,
                        void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || nseg < 1 || (seg_off == nullptr && nseg != 1)) return CO3_EINVAL;
    if (!chunk_ok(chunk_syms) || cap_words < 0 || cap_words % 2 != 0) return CO3_EINVAL;
    if (!g || !err || !anchor || !counts || !codes || !words || !chunk_bitoff || !total_bits || !workspace)
        return CO3_EINVAL;
    if (!aligned(g, 16) || !aligned(err, 16) || !aligned(words, 16) || !aligned(codes, 8) || !aligned(workspace, 256))
        return CO3_EINVAL;
    if (sym && !aligned(sym, 16)) return CO3_EINVAL;
    if (ws_bytes < co3_user_encode_workspace_bytes(n, U, stride, nseg, sym != nullptr)) return CO3_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FmtC fc(fmt);
    char *ws = static_cast<char *>(workspace);
    void *enc_ws = ws;
    ws += round_up_256(co3_encode_workspace_bytes(n, U));
    uint8_t *symbuf = sym ? sym : reinterpret_cast<uint8_t *>(ws);
    if (!sym) ws += round_up_256((size_t)U * (size_t)(stride > n ? stride : n) + 16);
    // symbols that stay inside the call take four bits each where the alphabet allows
    const int nib = !sym && fc.K <= 16 && (U == 1 || stride % 2 == 0) ? 1 : 0;
    int kpt = 0, grid = 0;
    const bool coop = user_encode_coop(n, U, nseg, &kpt, &grid);
    uint32_t *counts_rep = nullptr;
    if (coop) {
        // exchange words [U][grid], with several tensors per user the tensors' maxima [U][nseg] behind them
        uint32_t *slots = reinterpret_cast<uint32_t *>(ws);
        const int64_t ntmax = nseg > 1 ? (int64_t)U * nseg : 0;
        uint32_t *tmax = nseg > 1 ? slots + (int64_t)U * grid : nullptr;
        ws += round_up_256(((size_t)U * (size_t)grid + (size_t)ntmax) * sizeof(uint32_t));
        counts_rep = reinterpret_cast<uint32_t *>(ws);
        // exchange words, maxima and partial counters start at zero
        if (co3_launch_fill(reinterpret_cast<int32_t *>(slots), (int64_t)U * grid + ntmax, 0, counts_rep,
                            (int64_t)CO3_COOP_COUNT_REPS * U * fc.K, st) != hipSuccess)
            return CO3_EHIP;
        if (co3_launch_coop_convert(g, err, symbuf, n, U, stride, kpt, grid, nseg > 1 ? seg_off : nullptr, nseg, anchor, gamma,
                                    fmt, counts_rep, slots, tmax, g_spin_limit.load(), status, nib, st) != hipSuccess)
            return CO3_EHIP;
    } else {
        const int32_t rc = convert_common(g, err, symbuf, n, U, stride, seg_off, nseg, anchor, CO3_ANCHOR_FROM_ABSMAX_G,
                                          nullptr, gamma, fmt, counts, stream, nib);
        if (rc != CO3_OK) return rc;
    }
    // the codes (after a resident grid: with the ragged end of the vector and the partial count tables added
    // up, in the same launch), then the compression
    const hipError_t e = coop ? co3_launch_user_finish(g, err, symbuf, n, co3_coop_full_elements(n, kpt), stride, U,
                                                       nseg > 1 ? seg_off : nullptr, nseg, anchor, gamma, fmt, nib, counts_rep, CO3_COOP_COUNT_REPS, counts, codes, status, st, 0, U)
                              : co3_launch_build_code(counts, U, fc.K, codes, status, st);
    if (e != hipSuccess) return CO3_EHIP;
    return hip_rc(co3_launch_encode(symbuf, n, U, stride, codes, fc.K, nullptr, 1, words, cap_words, chunk_syms, chunk_bitoff,
                                    total_bits, static_cast<uint64_t *>(enc_ws), status, st, nib));
}

int32_t co3_moments(const float *g, const float *err, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                    int32_t nseg, float gamma, double *sums, void *stream)
{
    if (!batch_ok(n, U, stride) || nseg < 1 || (seg_off == nullptr && nseg != 1)) return CO3_EINVAL;
    if (!g || !err || !sums || !aligned(g, 16) || !aligned(err, 16) || !aligned(sums, 8)) return CO3_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the sums start at +0.0: all-zero bits
    hipError_t e = co3_launch_fill(reinterpret_cast<int32_t *>(sums), (int64_t)U * nseg * 4, 0, nullptr, 0, st);
    if (e != hipSuccess) return CO3_EHIP;
    return hip_rc(co3_launch_moments(g, err, n, U, stride, seg_off, nseg, gamma, sums, st));
}

int32_t co3_bias_scale(const double *sums, int64_t n, int32_t U, const int64_t *seg_off, int32_t nseg, float *scale,
                       double *fit, void *stream)
{
    if (n < 0 || U < 1 || nseg < 1 || (seg_off == nullptr && nseg != 1) || !sums || !scale) return CO3_EINVAL;
    return hip_rc(co3_launch_bias_scale(sums, n, U, seg_off, nseg, scale, fit, static_cast<hipStream_t>(stream)));
}

int32_t co3_histogram(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, uint32_t *counts,
                      void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || !sym || !counts || !aligned(sym, 16)) return CO3_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FmtC fc(fmt);
    hipError_t e = co3_launch_fill(nullptr, 0, 0, counts, (int64_t)U * fc.K, st);
    if (e != hipSuccess) return CO3_EHIP;
    return hip_rc(co3_launch_histogram(sym, n, U, stride, fc.K, counts, st));
}

int32_t co3_build_code(const uint32_t *weights, int32_t U, co3_fmt fmt, void *codes, int32_t *status, void *stream)
{
    if (!fmt_ok(fmt) || U < 1 || !weights || !codes || !aligned(codes, 8)) return CO3_EINVAL;
    const FmtC fc(fmt);
    return hip_rc(co3_launch_build_code(weights, U, fc.K, codes, status, static_cast<hipStream_t>(stream)));
}

static int32_t encode_common(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                             const int64_t *seg_off, int32_t nseg, uint64_t *words, int64_t cap_words,
                             int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits, void *workspace,
                             size_t ws_bytes, int32_t *status, void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || !chunk_ok(chunk_syms) || cap_words < 0) return CO3_EINVAL;
    if (!sym || !codes || !words || !chunk_bitoff || !total_bits || !workspace) return CO3_EINVAL;
    if (!aligned(sym, 16) || !aligned(words, 16) || !aligned(codes, 8) || !aligned(workspace, 8)) return CO3_EINVAL;
    if (cap_words % 2 != 0) return CO3_EINVAL;
    if (ws_bytes < co3_encode_workspace_bytes(n, U)) return CO3_EINVAL;
    const FmtC fc(fmt);
    return hip_rc(co3_launch_encode(sym, n, U, stride, codes, fc.K, seg_off, nseg, words, cap_words, chunk_syms,
                                    chunk_bitoff, total_bits, static_cast<uint64_t *>(workspace), status,
                                    static_cast<hipStream_t>(stream)));
}

int32_t co3_encode(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                   uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                   uint64_t *total_bits, void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    return encode_common(sym, n, U, stride, fmt, codes, nullptr, 1, words, cap_words, chunk_syms, chunk_bitoff,
                         total_bits, workspace, ws_bytes, status, stream);
}

int32_t co3_encode_static(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                          uint64_t *words, int64_t cap_words, int32_t chunk_syms, uint64_t *chunk_bitoff,
                          uint64_t *total_bits, int32_t *status, void *stream)
{
    // sizes first: nothing of the runtime is touched for a batch that the fixed workspace cannot serve
    if (n < 0 || U < 1) return CO3_EINVAL;
    const size_t need = co3_encode_workspace_bytes(n, U);
    if (need > (size_t)CO3_ENCODE_STATIC_WS_BYTES) return CO3_EINVAL;
    void *ws = nullptr;
    if (co3_static_encode_workspace(&ws) != hipSuccess) return CO3_EHIP;
    return encode_common(sym, n, U, stride, fmt, codes, nullptr, 1, words, cap_words, chunk_syms, chunk_bitoff,
                         total_bits, ws, need, status, stream);
}

int32_t co3_encode_layers(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, co3_fmt fmt, const void *codes,
                          const int64_t *seg_off, int32_t nseg, uint64_t *words, int64_t cap_words,
                          int32_t chunk_syms, uint64_t *chunk_bitoff, uint64_t *total_bits, void *workspace,
                          size_t ws_bytes, int32_t *status, void *stream)
{
    if (!seg_off || nseg < 1) return CO3_EINVAL;
    return encode_common(sym, n, U, stride, fmt, codes, seg_off, nseg, words, cap_words, chunk_syms, chunk_bitoff,
                         total_bits, workspace, ws_bytes, status, stream);
}

int32_t co3_histogram_layers(const uint8_t *sym, int64_t n, int32_t U, int64_t stride, const int64_t *seg_off,
                             int32_t nseg, co3_fmt fmt, int32_t pool_users, uint32_t *counts, void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || !sym || !counts || !aligned(sym, 16)) return CO3_EINVAL;
    if (!seg_off || nseg < 1) return CO3_EINVAL;
    if (pool_users && (int64_t)n * U >= ((int64_t)1 << 32)) return CO3_EINVAL;      // 32-bit counters summed over the users
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FmtC fc(fmt);
    hipError_t e = co3_launch_fill(nullptr, 0, 0, counts, (int64_t)(pool_users ? 1 : U) * nseg * fc.K, st);
    if (e != hipSuccess) return CO3_EHIP;
    return hip_rc(co3_launch_histogram_layers(sym, n, U, stride, fc.K, seg_off, nseg, pool_users != 0, counts, st));
}

static int32_t decode_common(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                             const void *codes, const int64_t *code_seg_off, int32_t code_nseg, co3_fmt fmt, int64_t n,
                             int32_t U, uint8_t *sym_out, int64_t stride, int32_t *status, void *stream)
{
    if (!fmt_ok(fmt) || !batch_ok(n, U, stride) || !chunk_ok(chunk_syms) || cap_words < 0) return CO3_EINVAL;
    if (!words || !chunk_bitoff || !codes || !sym_out) return CO3_EINVAL;
    if (!aligned(sym_out, 16) || !aligned(words, 16) || !aligned(codes, 8) || cap_words % 2 != 0) return CO3_EINVAL;
    return hip_rc(co3_launch_decode(words, cap_words, chunk_bitoff, chunk_syms, codes, code_seg_off, code_nseg,
                                    FmtC(fmt).K, n, U, sym_out, stride, 0, status, static_cast<hipStream_t>(stream)));
}

int32_t co3_decode(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                   const void *codes, co3_fmt fmt, int64_t n, int32_t U, uint8_t *sym_out, int64_t stride,
                   int32_t *status, void *stream)
{
    return decode_common(words, cap_words, chunk_bitoff, chunk_syms, codes, nullptr, 1, fmt, n, U, sym_out, stride,
                         status, stream);
}

int32_t co3_decode_layers(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                          const void *codes, const int64_t *seg_off, int32_t nseg, co3_fmt fmt, int64_t n, int32_t U,
                          uint8_t *sym_out, int64_t stride, int32_t *status, void *stream)
{
    if (!seg_off || nseg < 1) return CO3_EINVAL;
    return decode_common(words, cap_words, chunk_bitoff, chunk_syms, codes, seg_off, nseg, fmt, n, U, sym_out, stride,
                         status, stream);
}

// code_seg_off != NULL: codes holds one code per code group [code_seg_off[s], code_seg_off[s+1]) shared by the
// users, instead of one code per user
static int32_t aggregate_common(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                int32_t chunk_syms, const void *codes, const int64_t *code_seg_off, int32_t code_nseg,
                                co3_fmt fmt, int64_t n, int32_t U, const int32_t *anchor, const float *scale,
                                const int64_t *seg_off, int32_t nseg, float *avg_out, void *workspace, size_t ws_bytes,
                                int32_t *status, void *stream, const float *acc_in = nullptr, int32_t divide_by = -1)
{
    if (!fmt_ok(fmt) || n < 0 || n >= ((int64_t)1 << 32) || U < 1 || !chunk_ok(chunk_syms) || cap_words < 0)
        return CO3_EINVAL;
    if (acc_in && !aligned(acc_in, 16)) return CO3_EINVAL;
    const float divisor = divide_by < 0 ? (float)U : (float)divide_by;      // 0: the sum is left undivided
    if (nseg < 1 || (seg_off == nullptr && nseg != 1) || code_nseg < 1) return CO3_EINVAL;
    if (!words || !chunk_bitoff || !codes || !anchor || !avg_out || !workspace) return CO3_EINVAL;
    if (!aligned(avg_out, 16) || !aligned(workspace, 16) || !aligned(words, 16) || !aligned(codes, 8)) return CO3_EINVAL;
    if (cap_words % 2 != 0) return CO3_EINVAL;
    const size_t need = co3_ps_aggregate_workspace_bytes(n, U, chunk_syms);
    if (ws_bytes < need) return CO3_EINVAL;
    const int64_t ws_stride = (int64_t)(need / (size_t)U);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *symws = static_cast<uint8_t *>(workspace);
    hipError_t e = co3_launch_decode(words, cap_words, chunk_bitoff, chunk_syms, codes, code_seg_off, code_nseg,
                                     FmtC(fmt).K, n, U, symws, ws_stride, 1, status, st);
    if (e != hipSuccess) return CO3_EHIP;
    const int packed = co3_ws_packed(FmtC(fmt).K, chunk_syms, code_seg_off ? code_nseg : 0) ? 1 : 0;
    return hip_rc(co3_launch_ps_sum_tiled(symws, n, U, ws_stride, chunk_syms, anchor, scale, seg_off, nseg, fmt, packed,
                                          acc_in, divisor, avg_out, st));
}

int32_t co3_ps_aggregate(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                         const void *codes, co3_fmt fmt, int64_t n, int32_t U, const int32_t *anchor,
                         const int64_t *seg_off, int32_t nseg, float *avg_out, void *workspace, size_t ws_bytes,
                         int32_t *status, void *stream)
{
    return aggregate_common(words, cap_words, chunk_bitoff, chunk_syms, codes, nullptr, 1, fmt, n, U, anchor, nullptr,
                            seg_off, nseg, avg_out, workspace, ws_bytes, status, stream);
}

int32_t co3_ps_aggregate_partial(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                 int32_t chunk_syms, const void *codes, co3_fmt fmt, int64_t n, int32_t U,
                                 const int32_t *anchor, const int64_t *seg_off, int32_t nseg, const float *acc_in,
                                 int32_t divide_by, float *out, void *workspace, size_t ws_bytes, int32_t *status,
                                 void *stream)
{
    if (divide_by < 0) return CO3_EINVAL;
    return aggregate_common(words, cap_words, chunk_bitoff, chunk_syms, codes, nullptr, 1, fmt, n, U, anchor, nullptr,
                            seg_off, nseg, out, workspace, ws_bytes, status, stream, acc_in, divide_by);
}

int32_t co3_ps_decode_users(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff, int32_t chunk_syms,
                            const void *codes, co3_fmt fmt, int64_t n, int32_t U, int32_t first_user, int32_t U_total,
                            void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!fmt_ok(fmt) || n < 0 || n >= ((int64_t)1 << 32) || U < 1 || !chunk_ok(chunk_syms) || cap_words < 0 || cap_words % 2)
        return CO3_EINVAL;
    if (first_user < 0 || U_total < 1 || first_user + U > U_total) return CO3_EINVAL;
    if (!words || !chunk_bitoff || !codes || !workspace) return CO3_EINVAL;
    if (!aligned(workspace, 16) || !aligned(words, 16) || !aligned(codes, 8)) return CO3_EINVAL;
    const size_t need = co3_ps_aggregate_workspace_bytes(n, U_total, chunk_syms);
    if (ws_bytes < need) return CO3_EINVAL;
    const int64_t ws_stride = (int64_t)(need / (size_t)U_total);
    uint8_t *symws = static_cast<uint8_t *>(workspace) + (size_t)first_user * (size_t)ws_stride;
    return hip_rc(co3_launch_decode(words, cap_words, chunk_bitoff, chunk_syms, codes, nullptr, 1, FmtC(fmt).K, n, U, symws,
                                    ws_stride, 1, status, static_cast<hipStream_t>(stream)));
}

int32_t co3_ps_average(const void *workspace, size_t ws_bytes, int32_t chunk_syms, co3_fmt fmt, int64_t n, int32_t U,
                       const int32_t *anchor, const int64_t *seg_off, int32_t nseg, float *avg_out, void *stream)
{
    if (!fmt_ok(fmt) || n < 0 || n >= ((int64_t)1 << 32) || U < 1 || !chunk_ok(chunk_syms)) return CO3_EINVAL;
    if (nseg < 1 || (seg_off == nullptr && nseg != 1)) return CO3_EINVAL;
    if (!workspace || !anchor || !avg_out || !aligned(workspace, 16) || !aligned(avg_out, 16)) return CO3_EINVAL;
    const size_t need = co3_ps_aggregate_workspace_bytes(n, U, chunk_syms);
    if (ws_bytes < need) return CO3_EINVAL;
    const int packed = co3_ws_packed(FmtC(fmt).K, chunk_syms, 0) ? 1 : 0;
    return hip_rc(co3_launch_ps_sum_tiled(static_cast<const uint8_t *>(workspace), n, U, (int64_t)(need / (size_t)U), chunk_syms,
                                          anchor, nullptr, seg_off, nseg, fmt, packed, nullptr, (float)U, avg_out,
                                          static_cast<hipStream_t>(stream)));
}

int32_t co3_ps_aggregate_scaled(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                int32_t chunk_syms, const void *codes, co3_fmt fmt, int64_t n, int32_t U,
                                const int32_t *anchor, const float *scale, const int64_t *seg_off, int32_t nseg,
                                float *avg_out, void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!scale) return CO3_EINVAL;
    return aggregate_common(words, cap_words, chunk_bitoff, chunk_syms, codes, nullptr, 1, fmt, n, U, anchor, scale,
                            seg_off, nseg, avg_out, workspace, ws_bytes, status, stream);
}

int32_t co3_ps_aggregate_layers(const uint64_t *words, int64_t cap_words, const uint64_t *chunk_bitoff,
                                int32_t chunk_syms, const void *codes, const int64_t *code_seg_off, int32_t code_nseg,
                                co3_fmt fmt, int64_t n, int32_t U, const int32_t *anchor, const float *scale,
                                const int64_t *seg_off, int32_t nseg, float *avg_out, void *workspace, size_t ws_bytes,
                                int32_t *status, void *stream)
{
    if (!code_seg_off) return CO3_EINVAL;
    return aggregate_common(words, cap_words, chunk_bitoff, chunk_syms, codes, code_seg_off, code_nseg, fmt, n, U,
                            anchor, scale, seg_off, nseg, avg_out, workspace, ws_bytes, status, stream);
}

// ---- model table (host arithmetic only) ---------------------------------------------------

// Regularised lower incomplete gamma function P(a, x), a > 0, x >= 0: power series for x < a + 1,
// continued fraction for the complement otherwise.
static double reg_lower_gamma(double a, double x)
{
    if (!(x > 0.0)) return 0.0;
    if (isinf(x)) return 1.0;
    const double lg = lgamma(a);
    if (x < a + 1.0) {
        double term = 1.0 / a, sum = term, ap = a;
        for (int it = 0; it < 100000; ++it) {
            ap += 1.0;
            term *= x / ap;
            sum += term;
            if (fabs(term) < fabs(sum) * 1e-17) break;
        }
        return sum * exp(-x + a * log(x) - lg);
    }
    const double tiny = 1e-300;
    double b = x + 1.0 - a, c = 1.0 / tiny, d = 1.0 / b, h = d;
    for (int it = 1; it < 100000; ++it) {
        double an = -(double)it * ((double)it - a);
        b += 2.0;
        d = an * d + b;
        if (fabs(d) < tiny) d = tiny;
        c = b + an / c;
        if (fabs(c) < tiny) c = tiny;
        d = 1.0 / d;
        double delta = d * c;
        h *= delta;
        if (fabs(delta - 1.0) < 1e-16) break;
    }
    double qv = exp(-x + a * log(x) - lg) * h;
    return 1.0 - qv;
}

static double gennorm_cdf_pos(double x, double beta, double alpha)   // x >= 0
{
    return 0.5 + 0.5 * reg_lower_gamma(1.0 / beta, pow(x / alpha, beta));
}

int32_t co3_model_weights(int32_t A, co3_fmt fmt, double beta, double alpha, uint32_t *weights_host)
{
    if (!fmt_ok(fmt) || !weights_host || !(beta > 0.0) || !(alpha > 0.0)) return CO3_EINVAL;
    const FmtC fc(fmt);
    const int half = fc.K / 2;
    const int e_min = A - fc.F + 1;
    double mags[128];
    for (int c = 0; c < half; ++c) {
        int f = c >> fc.M, m = c & ((1 << fc.M) - 1);
        double frac = (double)m / (double)(1 << fc.M);
        mags[c] = f ? ldexp(1.0 + frac, e_min + f - 1) : ldexp(frac, e_min);
    }
    for (int c = 0; c < half; ++c) {
        double lo = c ? 0.5 * (mags[c - 1] + mags[c]) : 0.0;
        double cdf_lo = gennorm_cdf_pos(lo, beta, alpha);
        double cdf_hi = (c + 1 < half) ? gennorm_cdf_pos(0.5 * (mags[c] + mags[c + 1]), beta, alpha) : 1.0;
        double p = cdf_hi - cdf_lo;
        if (c == 0) p *= 2.0;      // the zero cell is symmetric about 0
        double w = nearbyint(p * 4294967296.0);
        if (!(w >= 1.0)) w = 1.0;
        if (w > 4294967295.0) w = 4294967295.0;
        weights_host[c] = (uint32_t)w;
        weights_host[half + c] = c ? (uint32_t)w : 0u;
    }
    return CO3_OK;
}

int32_t co3_design_layer_tables(const double *fit, const float *scale, int32_t U, int32_t nseg, const int64_t *seg_off,
                                const int64_t *code_seg_off, int32_t ncodes, int32_t A, co3_fmt fmt,
                                uint32_t *weights_host)
{
    if (!fmt_ok(fmt) || !fit || !scale || !seg_off || !code_seg_off || !weights_host || U < 1 || nseg < 1 || ncodes < 1)
        return CO3_EINVAL;
    const int K = 1 << (1 + fmt.exp_bits + fmt.mant_bits);
    for (int k = 0; k < ncodes; ++k) {
        const int64_t a = code_seg_off[k], b = code_seg_off[k + 1];
        int s_best = -1;
        int64_t size_best = 0;
        int s_holds = 0;                                  // tensor that holds the group's first element
        for (int s = 0; s < nseg; ++s) {
            const int64_t size = seg_off[s + 1] - seg_off[s];
            if (seg_off[s] <= a && a < seg_off[s + 1]) s_holds = s;
            if (seg_off[s] >= a && seg_off[s] < b && size > size_best) {
                s_best = s;
                size_best = size;
            }
        }
        const int s = s_best >= 0 ? s_best : s_holds;
        double beta = 0.0, alpha = 0.0;
        for (int u = 0; u < U; ++u) {
            const size_t j = (size_t)u * nseg + s;
            beta += fit[2 * j];
            alpha += fit[2 * j + 1] * (double)scale[j];
        }
        beta /= (double)U;
        alpha /= (double)U;
        beta = beta < 0.2 ? 0.2 : beta > 4.0 ? 4.0 : beta;
        alpha = alpha < 1e-30 ? 1e-30 : alpha;
        if (!(beta == beta) || !(alpha == alpha)) return CO3_EINVAL;          // a fit that is not a number
        const int32_t rc = co3_model_weights(A, fmt, beta, alpha, weights_host + (size_t)k * K);
        if (rc != CO3_OK) return rc;
    }
    return CO3_OK;
}

}  // extern "C"
