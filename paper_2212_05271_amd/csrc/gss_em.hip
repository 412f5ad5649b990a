// Guided cACGMM EM (arXiv 2212.05271, Section 2.2, Eq. (2)-(5)) for gfx950.
//
// One EM iteration = M-step (class scatter matrices B_{f,k} and weights pi_{f,k} from the posteriors)
// followed by an E-step (posteriors from Eq. (3)-(5)).  The E-step that ends iteration i and the M-step
// that starts iteration i+1 use the same quadratic forms q = y^H B^-1 y, so they are fused into one
// pass over Y:
//
//   pass i (i = 0 .. iters):   per frame: q_k, posterior gamma_k, weight w_k = gamma_k / q_k;
//                              i < iters: accumulate R_k = sum_t w_k y y^H, N_k = sum_t gamma_k
//                              i = iters: write gamma
//   factor i (i = 1 .. iters): B_k from (R_k, N_k), regularise, invert, log-det -> coefficients for pass i
//
// Pass 0 runs with B = I and uniform weights, which reproduces the initial posteriors
// gamma^0 = activity / (number of active classes) and q^0 = 1.
//
// Arithmetic.  The quadratic form is evaluated as the real inner product <B^-1, y y^H> over the D*D real
// degrees of freedom of the Hermitian outer product.  That form cancels heavily when B is
// ill-conditioned, so the outer product, the inner product and the scatter accumulation are done in
// fp64 from the RAW fp32 observations (products of fp32 numbers are exact in fp64); the unit
// normalisation of Eq. (2) is applied to q afterwards (q is homogeneous of degree 2 in y) and cancels
// in the M-step weight.  On this chip fp64 FMA issues at the same rate as unpacked fp32 FMA, so this
// costs registers, not time.  The posterior is fp64 as well, evaluated as pi_k / det B_k * q_k^-D in
// mantissa / exponent form (no logarithm, no exponential); only the gamma that leaves the library is
// rounded to fp32.
#include "gss_internal.h"

typedef int (*em_small_fn)(gss_ctx*, const gss_yview&, const uint8_t*, const int32_t*, int, int, int, int, int, float*,
                           hipStream_t);
#define GSS_DECL(DD, KK)                                                                                          \
  int gss_em_small_d##DD##_k##KK(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity, const int32_t* T_len, int S, \
                                 int F, int Tmax, int iters, int weight_mode, float* gamma, hipStream_t st);
#define GSS_DECL_ROW(DD) \
  GSS_DECL(DD, 1) GSS_DECL(DD, 2) GSS_DECL(DD, 3) GSS_DECL(DD, 4) GSS_DECL(DD, 5) GSS_DECL(DD, 6) GSS_DECL(DD, 7) GSS_DECL(DD, 8)
GSS_DECL_ROW(1) GSS_DECL_ROW(2) GSS_DECL_ROW(3) GSS_DECL_ROW(4) GSS_DECL_ROW(5) GSS_DECL_ROW(6) GSS_DECL_ROW(7) GSS_DECL_ROW(8)
#undef GSS_DECL_ROW
#undef GSS_DECL

#define GSS_ROW(DD)                                                                                               \
  { gss_em_small_d##DD##_k1, gss_em_small_d##DD##_k2, gss_em_small_d##DD##_k3, gss_em_small_d##DD##_k4,          \
    gss_em_small_d##DD##_k5, gss_em_small_d##DD##_k6, gss_em_small_d##DD##_k7, gss_em_small_d##DD##_k8 }
static const em_small_fn kEmSmall[8][8] = {GSS_ROW(1), GSS_ROW(2), GSS_ROW(3), GSS_ROW(4),
                                           GSS_ROW(5), GSS_ROW(6), GSS_ROW(7), GSS_ROW(8)};
#undef GSS_ROW

static int em_dispatch(gss_ctx* ctx, const gss_yview& yv, const uint8_t* activity, const int32_t* T_len, int S, int F,
                       int Tmax, int D, int K, int iters, int weight_mode, float* gamma, void* stream) {
  if (S <= 0 || F <= 0 || Tmax <= 0 || D <= 0 || K <= 0 || iters < 0) return GSS_EINVAL;
  if (weight_mode != 0 && weight_mode != 1) return GSS_EINVAL;
  if (D > GSS_MAX_D || K > GSS_MAX_K) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  hipStream_t st = (hipStream_t)stream;
  if (D <= 8) return kEmSmall[D - 1][K - 1](ctx, yv, activity, T_len, S, F, Tmax, iters, weight_mode, gamma, st);
  return gss_em_large(ctx, yv, activity, T_len, S, F, Tmax, D, K, iters, weight_mode, gamma, st);
}

extern "C" int gss_cacgmm_em(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                             int S, int F, int Tmax, int D, int K, int iters, int weight_mode,
                             float* gamma, void* stream) {
  if (!ctx || !Y || !activity || !gamma) return GSS_EINVAL;
  if (F <= 0 || Tmax <= 0 || D <= 0) return GSS_EINVAL;
  return em_dispatch(ctx, gss_dense_view(Y, F, Tmax, D), activity, T_len, S, F, Tmax, D, K, iters, weight_mode, gamma,
                     stream);
}

extern "C" int gss_cacgmm_em_frames(gss_ctx* ctx, const float* Yrec, int64_t Trec, const int64_t* frame0,
                                    const uint8_t* activity, const int32_t* T_len, int S, int F, int Tmax, int D,
                                    int K, int iters, int weight_mode, float* gamma, void* stream) {
  if (!ctx || !Yrec || !frame0 || !activity || !gamma) return GSS_EINVAL;
  if (Trec <= 0 || D <= 0) return GSS_EINVAL;
  return em_dispatch(ctx, gss_frames_view(Yrec, Trec, frame0, D), activity, T_len, S, F, Tmax, D, K, iters, weight_mode,
                     gamma, stream);
}
