/*
 * libgss: guided source separation (GSS) hot path for AMD MI355X (gfx950).
 *
 * The calls follow the problem statement of arXiv 2212.05271, Section 2:
 * multichannel STFT Y[f,t,:] in C^D plus binary speaker activities a[k,t]
 * -> cACGMM masks gamma[k,f,t] (Section 2.2) -> mask-based MVDR output
 * X[f,t] for one target class (Section 2.3), with the STFT and its inverse
 * around them (Section 3, the list of operations moved to the GPU).
 *
 * Conventions common to every entry point
 *   - Plain C ABI.  Pointers are DEVICE pointers unless the comment says "host".
 *   - The caller owns every input and output buffer.  The library owns only its
 *     context and the scratch memory inside it (grown on demand with hipMalloc,
 *     freed by gss_destroy).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising the host,
 *     except that growing the scratch memory synchronises the device once.
 *   - Calls that share one context must be issued on one stream (or be ordered
 *     by the caller): they share the context's scratch memory.
 *   - Return value: GSS_OK (0) or a negative gss_status.  Nothing is written on
 *     error.  The library never aborts and never writes outside the outputs.
 *   - Complex numbers are interleaved (re, im) float pairs ("complex64").
 *   - Layouts are C order, last index fastest.
 *   - D = number of channels, K = number of mixture classes INCLUDING the noise
 *     class (the noise class is simply a row of `activity` that is all ones),
 *     F = frequency bins, S = segments in the batch, Tmax = padded frame count.
 *   - T_len[s] (device, may be NULL = every segment has Tmax frames) gives the
 *     number of valid frames of segment s; outputs at t >= T_len[s] are exact 0.
 */
#ifndef GSS_H
#define GSS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gss_status {
  GSS_OK = 0,
  GSS_EINVAL = -1,       /* null pointer, non-positive size, out-of-range argument   */
  GSS_EUNSUPPORTED = -2, /* shape outside what the kernels are built for             */
  GSS_ENOMEM = -3,       /* scratch allocation failed                                */
  GSS_EHIP = -4,         /* the HIP runtime reported an error (launch, device, ...)  */
  GSS_ETOOBIG = -5       /* the problem needs more scratch than the fixed static buffer of a
                            no-allocation entry point holds (GSS_STATIC_SCRATCH_BYTES)          */
} gss_status;

/* Limits of the kernels in this build. */
#define GSS_MAX_D 32
#define GSS_MAX_K 8
#define GSS_WPE_MAX_D 8  /* gss_wpe: channels                                   */
#define GSS_WPE_MAX_N 80 /* gss_wpe: channels x taps (size of the linear system) */
#define GSS_WPE_LARGE_MAX_D 32  /* gss_wpe, large arrays: channels                  */
#define GSS_WPE_LARGE_MAX_N 320 /* gss_wpe, large arrays: channels x taps           */
#define GSS_STATIC_SCRATCH_BYTES (64u << 20) /* gss_cacgmm_em_noalloc: size of the static scratch array per GPU */

/* Bits of the device status word (gss_get_status). */
#define GSS_STATUS_NONPD_B 1u        /* a class scatter matrix had a non-positive pivot; the pivot was floored */
#define GSS_STATUS_NONPD_PHI 2u      /* the loaded background covariance had a non-positive pivot; floored     */
#define GSS_STATUS_BAD_TARGET 4u     /* a target index was outside [0, K); it was clamped                       */
#define GSS_STATUS_NONPD_WPE 8u      /* the loaded WPE correlation matrix had a non-positive pivot; floored     */
#define GSS_STATUS_ZERO_FRAME 16u    /* gss_cacgmm_em met a frame t < T_len[s] with ||y||^2 < 1e-20 (Eq. (2) is
                                        0/0 there): it was normalised to the zero vector, its q clamped        */
#define GSS_STATUS_BAD_REF 32u       /* a reference channel >= D was passed to gss_mvdr; it was chosen instead  */

typedef struct gss_ctx gss_ctx;

/* Create / destroy a context on HIP device `device_id`.  *out is set only on success. */
int gss_create(gss_ctx** out, int device_id);
void gss_destroy(gss_ctx* ctx);

/* Static, human-readable text for a gss_status value. */
const char* gss_strerror(int code);

/* Library version string ("major.minor.patch"), static storage. */
const char* gss_version(void);

/* Copies the device status word (OR of GSS_STATUS_* bits raised by earlier calls on this context)
 * to *host_out (host pointer) and clears it.  Synchronises `stream`. */
int gss_get_status(gss_ctx* ctx, uint32_t* host_out, void* stream);

/* Scratch bytes currently held by the context (host query, no device work). */
int64_t gss_scratch_bytes(const gss_ctx* ctx);

/*
 * Tuning options of a context (host call, no device work).  Returns GSS_EINVAL for an unknown option.
 *   GSS_OPT_EM_WHOLE_MIN_PROBLEMS: gss_cacgmm_em* runs a batch with at least this many (segment, frequency)
 *     problems (and D <= 8) in its one-wavefront-per-problem kernel, smaller batches in the kernels that cut a
 *     problem over several workgroups.  value < 0 restores the default (three problems per resident
 *     wavefront of the GPU); 0 always takes the one-wavefront-per-problem kernel.  Both give the same masks
 *     up to the order of the floating-point sums.
 */
#define GSS_OPT_EM_WHOLE_MIN_PROBLEMS 1
int gss_set_option(gss_ctx* ctx, int option, int64_t value);

/*
 * Per-kernel timing for measurements (not part of the method): when enabled, the launches of the
 * dominant kernels are bracketed with HIP events on the stream they are launched on.
 *   which = 0: the accumulating EM pass kernel (one launch per EM iteration)
 *   which = 1: the EM factor kernel (one launch per EM iteration)
 *   which = 2: the WPE covariance kernel (one launch per WPE iteration)
 * gss_profile_get waits for the recorded launches, returns their summed duration in milliseconds and
 * their count since the last call (both host pointers), and resets both.
 */
int gss_profile_enable(gss_ctx* ctx, int on);
int gss_profile_get(gss_ctx* ctx, int which, double* total_ms, int64_t* launches);

/*
 * STFT (Section 3 of the paper lists feature extraction among the operations run on the GPU; the paper
 * fixes only "513 bins", i.e. n_fft = 1024).
 *   x   [S][D][N] float32 time-domain samples
 *   Y   [S][F][T][D] complex64, F = n_fft/2 + 1, T = ceil(N / hop) + 3  (must equal the T passed in)
 * Periodic Hann window of n_fft samples; the signal is zero-padded by n_fft - hop samples on both
 * sides, so frame t covers samples [(t-3)*hop, (t+1)*hop).  Only n_fft = 1024, hop = 256 is built.
 * The first gss_stft or gss_istft call of a context allocates the context's twiddle table (4 KB) and
 * waits for `stream` once while it is filled.
 */
int gss_stft(gss_ctx* ctx, const float* x, int S, int D, int64_t N, int n_fft, int hop,
             float* Y, int T, void* stream);

/*
 * WPE dereverberation, independent per (segment, frequency): Section 2.1 removes the late reverberation
 * X^tail of its signal model with the weighted-prediction-error algorithm it cites (variance-normalised
 * delayed linear prediction) before the normalisation of Eq. (2).  With ytilde_t the stack of the `taps`
 * observations y_{t-delay}, y_{t-delay-1}, ... (D * taps components, zero before the first frame) and x = y
 * at the start, every iteration computes lambda_t = mean_d |x_{t,d}|^2 (floored at 1e-10 of its maximum
 * over the segment), R = sum_t ytilde_t ytilde_t^H / lambda_t, P = sum_t ytilde_t y_t^H / lambda_t,
 * G = (R + 1e-10 tr(R)/(D taps) I)^-1 P and x_t = y_t - G^H ytilde_t.
 *   Y      [S][F][Tmax][D] complex64
 *   T_len  [S] int32 or NULL: frames at t >= T_len[s] do not exist (no weight, nobody's past)
 *   taps >= 1, delay >= 1, iters >= 0 (0 copies the input); the usual setting is 10, 2, 3
 *   X      [S][F][Tmax][D] complex64 out, must not overlap Y; exact 0 at t >= T_len[s].  A bin that is
 *          silent, or too short for any frame to have a past, comes back unchanged.
 * Limits: D <= GSS_WPE_LARGE_MAX_D, D * taps <= GSS_WPE_LARGE_MAX_N, delay <= 64 (up to D = GSS_WPE_MAX_D and
 * D * taps = GSS_WPE_MAX_N the linear system of a frequency is solved in the registers of one workgroup, beyond
 * that by a blocked factorisation in global memory, which needs 16 * (D taps) * (D taps + D) bytes of scratch per
 * segment and frequency).  Arithmetic: fp64 throughout.
 */
int gss_wpe(gss_ctx* ctx, const float* Y, const int32_t* T_len, int S, int F, int Tmax, int D,
            int taps, int delay, int iters, float* X, void* stream);

/*
 * Guided cACGMM EM, independent per (segment, frequency): Eq. (2)-(5) and the EM loop of Section 2.2.
 *   Y        [S][F][Tmax][D] complex64, any scale (unit-normalised internally, Eq. (2))
 *   activity [S][K][Tmax] uint8, non-zero = class k may be active in frame t (a_{t,k} of Eq. (5))
 *   T_len    [S] int32 or NULL.  Segments of any mix of lengths go in one call: no work is done beyond a
 *            segment's own length, so grouping segments of similar length into separate calls saves only the
 *            memory of the padded arrays, not time
 *   iters    >= 0 EM iterations (each = M-step then E-step); 0 returns the normalised activity
 *   weight_mode  1: pi_{f,k} proportional to sum_t gamma; 0: pi uniform
 *   gamma    [S][K][F][Tmax] float32 out: the state posteriors after the last E-step = the masks.
 *            Exact 0 where activity is 0 and at t >= T_len[s].  The same bits on every run (all sums are taken
 *            in a fixed order).
 * Limits: 1 <= D <= GSS_MAX_D, 1 <= K <= GSS_MAX_K.
 */
int gss_cacgmm_em(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                  int S, int F, int Tmax, int D, int K, int iters, int weight_mode,
                  float* gamma, void* stream);

/*
 * gss_cacgmm_em on segments that are frame ranges of ONE recording's STFT (Section 2.2: a target segment is
 * processed together with a context window around it; Section 3, "Segment batching": the segments of a
 * recording are processed in batches).  Nothing is copied: segment s is the frames frame0[s] ..
 * frame0[s] + T_len[s] - 1 of the recording.
 *   Yrec   [F][Trec][D] complex64: STFT of the whole recording (gss_stft with S = 1)
 *   frame0 [S] int64 (device): first frame of every segment, 0 <= frame0[s] <= Trec
 *   T_len  [S] int32 (device) or NULL (= Tmax): frames of every segment; clipped to Tmax and to the frames the
 *          recording holds from frame0[s] on
 *   activity [S][K][Tmax], gamma [S][K][F][Tmax]: as for gss_cacgmm_em (indexed by the frame within the segment)
 * Everything else as for gss_cacgmm_em.
 */
int gss_cacgmm_em_frames(gss_ctx* ctx, const float* Yrec, int64_t Trec, const int64_t* frame0,
                         const uint8_t* activity, const int32_t* T_len, int S, int F, int Tmax, int D, int K,
                         int iters, int weight_mode, float* gamma, void* stream);

/*
 * gss_cacgmm_em for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc).  Same arguments, same kernels and same results as gss_cacgmm_em,
 * but the working memory (class coefficients and the partial sums of the M-step) lives in a static device
 * array of GSS_STATIC_SCRATCH_BYTES that the library holds once per GPU until the process ends; the call
 * makes no hipMalloc / hipFree and no other allocating call.
 *   - A problem whose working memory exceeds the array is rejected with GSS_ETOOBIG and nothing is written.
 *     The need is about 16 * S * F * K * D * D bytes (+ the partial sums of problems split over several
 *     workgroups when S * F is small): S * F * K * D * D <= 3.5 million always fits (e.g. 21 segments of
 *     513 bins at D = 8, K = 5).
 *   - Every call on one GPU, from any context, uses the same array: calls that overlap in time on one GPU
 *     race.  Order them on one stream or with events.  Nothing in the array has to survive between calls;
 *     each call initialises what it reads.
 */
int gss_cacgmm_em_noalloc(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                          int S, int F, int Tmax, int D, int K, int iters, int weight_mode,
                          float* gamma, void* stream);

/*
 * Mask-based MVDR (Souden form), Eq. (6)-(9) of Section 2.3, per segment and frequency.
 *   Y      [S][F][Tmax][D] complex64: used as handed over (NOT normalised inside)
 *   gamma  [S][K][F][Tmax] float32 masks
 *   target [S] int32: index of the class to extract, 0 <= target[s] < K (a value outside is clamped and
 *          raises GSS_STATUS_BAD_TARGET in the status word)
 *   ref    [S] int32 in/out: 0 <= ref[s] < D = use this reference channel; < 0 = choose the channel with
 *          the largest ratio of beamformed target power to beamformed background power summed over
 *          frequency (lowest index on ties); >= D is treated like < 0 and raises GSS_STATUS_BAD_REF; on
 *          return holds the channel used
 *   X      [S][F][Tmax] complex64 out: h(f)^H y_{t,f}; exact 0 at t >= T_len[s]
 */
int gss_mvdr(gss_ctx* ctx, const float* Y, const float* gamma, const int32_t* T_len,
             int S, int F, int Tmax, int D, int K, const int32_t* target, int32_t* ref,
             float* X, void* stream);

/*
 * gss_mvdr on segments that are frame ranges of one recording's STFT; Yrec, Trec, frame0, T_len as for
 * gss_cacgmm_em_frames, everything else as for gss_mvdr (Section 2.3, Eq. (6)-(9)).  X [S][F][Tmax].
 */
int gss_mvdr_frames(gss_ctx* ctx, const float* Yrec, int64_t Trec, const int64_t* frame0, const float* gamma,
                    const int32_t* T_len, int S, int F, int Tmax, int D, int K, const int32_t* target,
                    int32_t* ref, float* X, void* stream);

/*
 * The general form of gss_mvdr: dense batch or frame ranges of a recording, and the reference channel chosen per
 * segment or per frequency.  Section 3 ("Segment batching") notes that one reference channel for a whole batch
 * suits stationary speakers only; for speakers that move the channel may be chosen for every frequency on its own.
 *   Y, Trec, frame0 : Trec = 0 and frame0 = NULL: Y is a dense batch [S][F][Tmax][D] (as gss_mvdr);
 *                     Trec > 0 and frame0 != NULL: Y is a recording's STFT [F][Trec][D] (as gss_mvdr_frames)
 *   ref_mode = GSS_REF_PER_SEGMENT  : ref [S], as gss_mvdr
 *   ref_mode = GSS_REF_PER_FREQUENCY: ref [S][F] in/out; an entry < 0 (or >= D, flagged) is replaced by the channel
 *                     with the largest ratio of beamformed target power to beamformed background power at that
 *                     frequency (lowest index on ties); X[s][f][:] uses the filter of ref[s][f]
 */
#define GSS_REF_PER_SEGMENT 0
#define GSS_REF_PER_FREQUENCY 1
int gss_mvdr_ex(gss_ctx* ctx, const float* Y, int64_t Trec, const int64_t* frame0, const float* gamma,
                const int32_t* T_len, int S, int F, int Tmax, int D, int K, const int32_t* target,
                int ref_mode, int32_t* ref, float* X, void* stream);

/*
 * Inverse STFT matching gss_stft: inverse real FFT, synthesis window w / sum_shifts(w^2), overlap-add,
 * padding stripped.
 *   X  [S][F][T] complex64   (F = n_fft/2 + 1)
 *   x  [S][N] float32 out, with ceil(N / hop) + 3 == T
 */
int gss_istft(gss_ctx* ctx, const float* X, int S, int T, int n_fft, int hop,
              float* x, int64_t N, void* stream);

/*
 * Segment + context -> sample span and frame range (host, integers only; Section 2.2 "context window",
 * Section 3 item (ii)).  All pointers are HOST pointers.
 *   seg_start/seg_end [n_seg] target segment [start, end) in samples of a recording of n_samples
 *   ctx_left/ctx_right  context in samples added before / after (clipped to the recording)
 * Outputs, each [n_seg] (any may be NULL):
 *   ext_start, ext_end : the extended span snapped outward to multiples of hop (clipped to the
 *                        hop-rounded recording length)
 *   frame0, n_frames   : its frames in the recording's STFT (gss_stft numbering);
 *                        n_frames = (ext_end - ext_start)/hop + 3
 *   cut_start, cut_end : the target region as sample offsets inside the inverse STFT of those frames
 */
int gss_frames_from_segments(const int64_t* seg_start, const int64_t* seg_end, int n_seg,
                             int64_t n_samples, int64_t ctx_left, int64_t ctx_right, int hop,
                             int64_t* ext_start, int64_t* ext_end, int64_t* frame0, int32_t* n_frames,
                             int64_t* cut_start, int64_t* cut_end);

/*
 * Frame-level activity from sample-level activity (host, integers only).
 *   act_samples [K][n_samples] uint8 (host); frame t of the recording is centred on sample (t-1)*hop,
 *   clamped into the recording; out [K][n_frames] uint8 (host) for frames frame0 .. frame0+n_frames-1.
 */
int gss_frame_activity(const uint8_t* act_samples, int K, int64_t n_samples, int64_t frame0,
                       int32_t n_frames, int hop, uint8_t* out);

#ifdef __cplusplus
}
#endif
#endif /* GSS_H */
