// Internal declarations shared by the translation units of libgss (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gss.h"

// Constants of the algorithm (regularisation and guards).  The paper is silent on all of them; they are
// part of the algorithm's definition and are documented with the readings of the paper.
#define GSS_EPS_NORM_SQ 1e-20   // floor on ||y||^2 in the unit normalisation, Eq. (2)
#define GSS_EPS_N 1e-10         // floor on sum_t gamma and on a trace
#define GSS_EPS_Q 1e-10         // floor on y^H B^-1 y, Eq. (4)
#define GSS_EPS_PI 1e-30        // floor inside log(pi)
#define GSS_DELTA 1e-6          // diagonal loading of B (after scaling to trace D)
#define GSS_DELTA_BF 1e-6       // relative diagonal loading of Phi_bg
#define GSS_EPS_TRACE 1e-20     // added to Re tr(Phi_bg^-1 Phi_k), Eq. (8)
#define GSS_EPS_SNR 1e-300      // floor on the background power in the reference-channel ratio

#define GSS_PROFILE_SLOTS 64
#define GSS_PROFILE_KERNELS 3     // 0: EM pass (accumulating), 1: EM factor, 2: WPE covariance

struct gss_ctx {
  int device;
  void* scratch;          // device
  size_t scratch_cap;
  int scratch_fixed;      // non-zero while a no-allocation entry point runs: `scratch` is then this device's static
                          // array and gss_ensure_scratch refuses to grow it
  void* static_scratch;   // device address of the library's static scratch array on this context's device
  uint32_t* status;       // device, one word
  int num_cu;
  int64_t em_whole_min_problems;   // GSS_OPT_EM_WHOLE_MIN_PROBLEMS (< 0: default)
  void* twiddles;         // device: exp(-2 pi i k / 1024), k = 0..512 (float2), filled by the first STFT/iSTFT call
  // optional per-kernel timing with HIP events (gss_profile_enable / gss_profile_get)
  int profile;
  hipEvent_t ev_start[GSS_PROFILE_KERNELS][GSS_PROFILE_SLOTS], ev_stop[GSS_PROFILE_KERNELS][GSS_PROFILE_SLOTS];
  int ev_used[GSS_PROFILE_KERNELS];
  double prof_ms[GSS_PROFILE_KERNELS];
  int64_t prof_launches[GSS_PROFILE_KERNELS];
};

// Where the observations of a batch live.  Frame t, channel d of (segment s, frequency f) is the complex number
//   base[s * s_stride + f * f_stride + ((frame0 ? frame0[s] : 0) + t) * D + d].
// A dense batch [S][F][Tmax][D] has s_stride = F * Tmax * D, f_stride = Tmax * D, frame0 = NULL; segments
// that are frame ranges of one recording STFT [F][Trec][D] have s_stride = 0, f_stride = Trec * D and
// frame0[s] (device) = first frame of segment s.  t_limit = frames per (segment, frequency) row of the
// underlying array (Tmax or Trec): the kernels never read at or beyond it.
struct gss_yview {
  const float2* base;
  long s_stride, f_stride;
  const int64_t* frame0;
  long t_limit;
};
static inline gss_yview gss_dense_view(const float* Y, int F, int Tmax, int D) {
  gss_yview v;
  v.base = (const float2*)Y;
  v.s_stride = (long)F * Tmax * D;
  v.f_stride = (long)Tmax * D;
  v.frame0 = nullptr;
  v.t_limit = Tmax;
  return v;
}
static inline gss_yview gss_frames_view(const float* Yrec, int64_t Trec, const int64_t* frame0, int D) {
  gss_yview v;
  v.base = (const float2*)Yrec;
  v.s_stride = 0;
  v.f_stride = (long)Trec * D;
  v.frame0 = frame0;
  v.t_limit = (long)Trec;
  return v;
}

// Brackets one kernel launch with HIP events on `st` when profiling is on.
void gss_profile_begin(gss_ctx* ctx, int which, hipStream_t st);
void gss_profile_end(gss_ctx* ctx, int which, hipStream_t st);

// Kernels for 9 <= D <= GSS_MAX_D channels (gss_large.hip), called by the entry points after validation.
int gss_em_large(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity, const int32_t* T_len, int S, int F, int Tmax,
                 int D, int K, int iters, int weight_mode, float* gamma, hipStream_t st);
int gss_mvdr_large(gss_ctx* ctx, const gss_yview& Y, const float* gamma, const int32_t* T_len, int S, int F, int Tmax,
                   int D, int K, const int32_t* target, int32_t* ref, int ref_per_f, float* X, hipStream_t st);
// Reference-channel kernel shared by the small- and large-D MVDR paths (gss_mvdr.hip).
void gss_launch_mvdr_ref(const double* pw, int32_t* ref, uint32_t* status, int S, int F, int D, int ref_per_f,
                         hipStream_t st);

// Makes sure ctx->scratch holds at least `bytes`.  Growing synchronises the device (the old block may
// still be in use by kernels already enqueued) and reallocates.  While ctx->scratch_fixed is set nothing is
// allocated: a request beyond the capacity returns GSS_ETOOBIG.
int gss_ensure_scratch(gss_ctx* ctx, size_t bytes);

static inline size_t gss_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#define GSS_HIP_CHECK(expr)                      \
  do {                                           \
    hipError_t e_ = (expr);                      \
    if (e_ != hipSuccess) return GSS_EHIP;       \
  } while (0)

// Packed real layout of a D x D Hermitian matrix used by the EM kernels, D*D reals in the order the
// per-frame outer product is generated:  for i = 0..D-1: [H_ii, then for j = i+1..D-1: Re H_ij, Im H_ij].
__host__ __device__ constexpr int gss_packed_row(int i, int D) { return 2 * i * D - i * i; }
