// One translation unit per class count K of the large-array EM kernels (compiled once for every
// GSS_INST_K = 1..8 by build.py).
#include "gss_large_impl.h"

#ifndef GSS_INST_K
#error "compile with -DGSS_INST_K=<classes>"
#endif

#define GSS_CAT2(a, b) a##b
#define GSS_CAT(a, b) GSS_CAT2(a, b)

int GSS_CAT(gss_em_large_k, GSS_INST_K)(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity, const int32_t* T_len,
                                        int S, int F, int Tmax, int D, int iters, int weight_mode, float* gamma,
                                        hipStream_t st) {
  return dispatch_nr<GSS_INST_K>(ctx, Y, activity, T_len, S, F, Tmax, D, iters, weight_mode, gamma, st);
}
