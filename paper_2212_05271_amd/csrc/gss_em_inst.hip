// One translation unit per (channel count D, class count K): compiled once for every GSS_INST_D = 1..8 and
// GSS_INST_K = 1..8 by build.py, so that the template instantiations compile in parallel.
#include "gss_em_impl.h"

#if !defined(GSS_INST_D) || !defined(GSS_INST_K)
#error "compile with -DGSS_INST_D=<channels> -DGSS_INST_K=<classes>"
#endif

#define GSS_CAT4(a, b, c, d) a##b##c##d
#define GSS_NAME(a, b, c, d) GSS_CAT4(a, b, c, d)

int GSS_NAME(gss_em_small_d, GSS_INST_D, _k, GSS_INST_K)(gss_ctx* ctx, const gss_yview& Y, const uint8_t* activity,
                                                          const int32_t* T_len, int S, int F, int Tmax, int iters,
                                                          int weight_mode, float* gamma, hipStream_t st) {
  return run_small<GSS_INST_D, GSS_INST_K>(ctx, Y, activity, T_len, S, F, Tmax, iters, weight_mode, gamma,
                                           st);
}
