// Entry points not built yet.
#include "gss_internal.h"
extern "C" {
int gss_stft(gss_ctx*, const float*, int, int, int64_t, int, int, float*, int, void*) { return GSS_EUNSUPPORTED; }
int gss_mvdr(gss_ctx*, const float*, const float*, const int32_t*, int, int, int, int, int, const int32_t*, int32_t*,
             float*, void*) { return GSS_EUNSUPPORTED; }
int gss_istft(gss_ctx*, const float*, int, int, int, int, float*, int64_t, void*) { return GSS_EUNSUPPORTED; }
}
