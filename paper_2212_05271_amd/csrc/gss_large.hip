// EM and MVDR kernels for large arrays, 9 <= D <= 32 channels (e.g. multi-array set-ups with 24
// microphones).  Same algorithm, same fp64 arithmetic and the same pass / factor structure as the D <= 8
// kernels (arXiv 2212.05271, Section 2.2 and 2.3); what changes is the mapping:
//
//   * D is a run-time value; the Hermitian outer product has M = D (D + 1) / 2 "items" (i <= j), each a
//     real diagonal entry or a complex off-diagonal one.  All per-class data is laid out per item:
//     coef[sf][m][k][2] (the two real coefficients that multiply Re and Im of item m), partial sums
//     part[sf][chunk][m][k][2].
//   * The frames of a tile sit in LDS as fp32 (exactly as they came), because D * 16 bytes of fp64 per
//     frame would not leave room for two workgroups per compute unit.
//   * Phase 1 (lane = frame) walks the items in a run-time loop, reading y_i, y_j of its own frame from
//     LDS and the class coefficients through the scalar path.
//   * Phase 2 (lane = a few items, frames in sequence): each lane owns NR items m = lane, lane + 64, ...,
//     forms them for every frame of the tile from LDS and accumulates K weighted sums per real part.
#include "gss_large_impl.h"

#define GSS_DECL_K(KK)                                                                                           \
  int gss_em_large_k##KK(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity, const int32_t* T_len, int S, int F, \
                         int Tmax, int D, int iters, int weight_mode, float* gamma, hipStream_t st);
GSS_DECL_K(1) GSS_DECL_K(2) GSS_DECL_K(3) GSS_DECL_K(4) GSS_DECL_K(5) GSS_DECL_K(6) GSS_DECL_K(7) GSS_DECL_K(8)
#undef GSS_DECL_K

int gss_em_large(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity, const int32_t* T_len, int S, int F, int Tmax,
                 int D, int K, int iters, int weight_mode, float* gamma, hipStream_t st) {
  switch (K) {
#define GSS_CASE_K(KK) \
  case KK: return gss_em_large_k##KK(ctx, Y, activity, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
    GSS_CASE_K(1) GSS_CASE_K(2) GSS_CASE_K(3) GSS_CASE_K(4) GSS_CASE_K(5) GSS_CASE_K(6) GSS_CASE_K(7) GSS_CASE_K(8)
#undef GSS_CASE_K
    default: return GSS_EUNSUPPORTED;
  }
}

int gss_mvdr_large(gss_ctx* ctx, const gss_yview& Y, const float* gamma, const int32_t* T_len, int S, int F, int Tmax,
                   int D, int K, const int32_t* target, int32_t* ref, int ref_per_f, float* X, hipStream_t st) {
  const gss_yview& Yc = Y;
  float2* Xc = (float2*)X;
  const int nr = (num_items(D) + kWave - 1) / kWave;
  if (nr <= 3) return run_mvdr_large<3>(ctx, Yc, gamma, T_len, S, F, Tmax, D, K, target, ref, ref_per_f, Xc, st);
  if (nr <= 5) return run_mvdr_large<5>(ctx, Yc, gamma, T_len, S, F, Tmax, D, K, target, ref, ref_per_f, Xc, st);
  if (nr <= 7) return run_mvdr_large<7>(ctx, Yc, gamma, T_len, S, F, Tmax, D, K, target, ref, ref_per_f, Xc, st);
  return run_mvdr_large<9>(ctx, Yc, gamma, T_len, S, F, Tmax, D, K, target, ref, ref_per_f, Xc, st);
}
