// One translation unit per channel count D (compiled once for every GSS_INST_D = 1..8 by build.py, so
// that the template instantiations over (D, K) compile in parallel).
#include "gss_em_impl.h"

#ifndef GSS_INST_D
#error "compile with -DGSS_INST_D=<channels>"
#endif

#define GSS_CAT2(a, b) a##b
#define GSS_CAT(a, b) GSS_CAT2(a, b)

int GSS_CAT(gss_em_small_d, GSS_INST_D)(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                                        int S, int F, int Tmax, int K, int iters, int weight_mode, float* gamma,
                                        hipStream_t st) {
  return dispatch_k<GSS_INST_D>(ctx, (const float2*)Y, activity, T_len, S, F, Tmax, K, iters, weight_mode, gamma, st);
}
