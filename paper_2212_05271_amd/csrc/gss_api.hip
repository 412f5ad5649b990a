// Context management, error strings and the host-side integer helpers of libgss.
#include "gss_internal.h"

#include <mutex>
#include <new>

// Working memory of gss_cacgmm_em_noalloc: one copy per GPU, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels and copies get the device address looked up below.
static __device__ __align__(256) unsigned char scratch[GSS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on `device` (which must be current), looked up once per device.
int static_scratch_address(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return GSS_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return GSS_EHIP;
    }
    g_static_ptr[device] = p;
  }
  *out = g_static_ptr[device];
  return GSS_OK;
}
}  // namespace

extern "C" {

const char* gss_version(void) { return "0.1.0"; }

const char* gss_strerror(int code) {
  switch (code) {
    case GSS_OK: return "ok";
    case GSS_EINVAL: return "invalid argument";
    case GSS_EUNSUPPORTED: return "shape not supported by this build";
    case GSS_ENOMEM: return "out of device memory";
    case GSS_EHIP: return "HIP runtime error";
    case GSS_ETOOBIG: return "problem exceeds the static scratch buffer of the no-allocation entry point";
    default: return "unknown error";
  }
}

int gss_create(gss_ctx** out, int device_id) {
  if (!out || device_id < 0) return GSS_EINVAL;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device_id >= n) return GSS_EHIP;
  GSS_HIP_CHECK(hipSetDevice(device_id));
  gss_ctx* c = new (std::nothrow) gss_ctx();
  if (!c) return GSS_ENOMEM;
  c->device = device_id;
  c->scratch = nullptr;
  c->scratch_cap = 0;
  c->scratch_fixed = 0;
  c->static_scratch = nullptr;
  c->status = nullptr;
  c->num_cu = 256;
  c->em_whole_min_problems = -1;
  c->twiddles = nullptr;
  c->profile = 0;
  for (int k = 0; k < GSS_PROFILE_KERNELS; ++k) {
    c->ev_used[k] = 0;
    c->prof_ms[k] = 0.0;
    c->prof_launches[k] = 0;
    for (int i = 0; i < GSS_PROFILE_SLOTS; ++i) { c->ev_start[k][i] = nullptr; c->ev_stop[k][i] = nullptr; }
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device_id) == hipSuccess && prop.multiProcessorCount > 0)
    c->num_cu = prop.multiProcessorCount;
  {
    const int rc = static_scratch_address(device_id, &c->static_scratch);
    if (rc != GSS_OK) {
      delete c;
      return rc;
    }
  }
  if (hipMalloc((void**)&c->status, sizeof(uint32_t)) != hipSuccess) {
    delete c;
    return GSS_ENOMEM;
  }
  if (hipMemset(c->status, 0, sizeof(uint32_t)) != hipSuccess) {
    (void)hipFree(c->status);
    delete c;
    return GSS_EHIP;
  }
  *out = c;
  return GSS_OK;
}

void gss_destroy(gss_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->device);
  (void)hipDeviceSynchronize();
  if (ctx->scratch) (void)hipFree(ctx->scratch);
  if (ctx->status) (void)hipFree(ctx->status);
  if (ctx->twiddles) (void)hipFree(ctx->twiddles);
  for (int k = 0; k < GSS_PROFILE_KERNELS; ++k)
    for (int i = 0; i < GSS_PROFILE_SLOTS; ++i) {
      if (ctx->ev_start[k][i]) (void)hipEventDestroy(ctx->ev_start[k][i]);
      if (ctx->ev_stop[k][i]) (void)hipEventDestroy(ctx->ev_stop[k][i]);
    }
  delete ctx;
}

int gss_get_status(gss_ctx* ctx, uint32_t* host_out, void* stream) {
  if (!ctx || !host_out) return GSS_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  GSS_HIP_CHECK(hipMemcpyAsync(host_out, ctx->status, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
  GSS_HIP_CHECK(hipStreamSynchronize(st));
  uint32_t zero = 0;
  GSS_HIP_CHECK(hipMemcpyAsync(ctx->status, &zero, sizeof(uint32_t), hipMemcpyHostToDevice, st));
  GSS_HIP_CHECK(hipStreamSynchronize(st));
  return GSS_OK;
}

int gss_cacgmm_em_noalloc(gss_ctx* ctx, const float* Y, const uint8_t* activity, const int32_t* T_len,
                          int S, int F, int Tmax, int D, int K, int iters, int weight_mode,
                          float* gamma, void* stream) {
  if (!ctx || !ctx->static_scratch) return GSS_EINVAL;
  // The kernels of gss_cacgmm_em take their working memory from ctx->scratch; for the duration of this call
  // that is the static array (by its device address), and growing it is refused.
  void* const saved = ctx->scratch;
  const size_t saved_cap = ctx->scratch_cap;
  ctx->scratch = ctx->static_scratch;
  ctx->scratch_cap = GSS_STATIC_SCRATCH_BYTES;
  ctx->scratch_fixed = 1;
  const int rc = gss_cacgmm_em(ctx, Y, activity, T_len, S, F, Tmax, D, K, iters, weight_mode, gamma, stream);
  ctx->scratch = saved;
  ctx->scratch_cap = saved_cap;
  ctx->scratch_fixed = 0;
  return rc;
}

int gss_set_option(gss_ctx* ctx, int option, int64_t value) {
  if (!ctx) return GSS_EINVAL;
  switch (option) {
    case GSS_OPT_EM_WHOLE_MIN_PROBLEMS:
      ctx->em_whole_min_problems = value;
      return GSS_OK;
    default:
      return GSS_EINVAL;
  }
}

int64_t gss_scratch_bytes(const gss_ctx* ctx) { return ctx ? (int64_t)ctx->scratch_cap : 0; }

int gss_profile_enable(gss_ctx* ctx, int on) {
  if (!ctx) return GSS_EINVAL;
  if (on) {
    if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
    for (int k = 0; k < GSS_PROFILE_KERNELS; ++k)
      for (int i = 0; i < GSS_PROFILE_SLOTS; ++i) {
        if (!ctx->ev_start[k][i]) GSS_HIP_CHECK(hipEventCreate(&ctx->ev_start[k][i]));
        if (!ctx->ev_stop[k][i]) GSS_HIP_CHECK(hipEventCreate(&ctx->ev_stop[k][i]));
      }
  }
  ctx->profile = on ? 1 : 0;
  return GSS_OK;
}

static int drain_profile(gss_ctx* ctx, int which) {
  for (int i = 0; i < ctx->ev_used[which]; ++i) {
    GSS_HIP_CHECK(hipEventSynchronize(ctx->ev_stop[which][i]));
    float ms = 0.f;
    GSS_HIP_CHECK(hipEventElapsedTime(&ms, ctx->ev_start[which][i], ctx->ev_stop[which][i]));
    ctx->prof_ms[which] += (double)ms;
    ctx->prof_launches[which] += 1;
  }
  ctx->ev_used[which] = 0;
  return GSS_OK;
}

int gss_profile_get(gss_ctx* ctx, int which, double* total_ms, int64_t* launches) {
  if (!ctx || which < 0 || which >= GSS_PROFILE_KERNELS || !total_ms || !launches) return GSS_EINVAL;
  int rc = drain_profile(ctx, which);
  if (rc != GSS_OK) return rc;
  *total_ms = ctx->prof_ms[which];
  *launches = ctx->prof_launches[which];
  ctx->prof_ms[which] = 0.0;
  ctx->prof_launches[which] = 0;
  return GSS_OK;
}

int gss_frames_from_segments(const int64_t* seg_start, const int64_t* seg_end, int n_seg,
                             int64_t n_samples, int64_t ctx_left, int64_t ctx_right, int hop,
                             int64_t* ext_start, int64_t* ext_end, int64_t* frame0, int32_t* n_frames,
                             int64_t* cut_start, int64_t* cut_end) {
  if (!seg_start || !seg_end || n_seg < 0 || n_samples <= 0 || hop <= 0 || ctx_left < 0 || ctx_right < 0)
    return GSS_EINVAL;
  const int64_t h = hop;
  const int64_t n_round = (n_samples + h - 1) / h * h;
  for (int i = 0; i < n_seg; ++i) {
    const int64_t s = seg_start[i], e = seg_end[i];
    if (s < 0 || e <= s || e > n_samples) return GSS_EINVAL;
  }
  for (int i = 0; i < n_seg; ++i) {
    const int64_t s = seg_start[i], e = seg_end[i];
    int64_t a = s - ctx_left;
    if (a < 0) a = 0;
    int64_t b = e + ctx_right;
    if (b > n_samples) b = n_samples;
    const int64_t es = a / h * h;
    int64_t ee = (b + h - 1) / h * h;
    if (ee > n_round) ee = n_round;
    if (ext_start) ext_start[i] = es;
    if (ext_end) ext_end[i] = ee;
    if (frame0) frame0[i] = es / h;
    if (n_frames) n_frames[i] = (int32_t)((ee - es) / h + 3);
    if (cut_start) cut_start[i] = s - es;
    if (cut_end) cut_end[i] = e - es;
  }
  return GSS_OK;
}

int gss_frame_activity(const uint8_t* act_samples, int K, int64_t n_samples, int64_t frame0,
                       int32_t n_frames, int hop, uint8_t* out) {
  if (!act_samples || !out || K <= 0 || n_samples <= 0 || n_frames < 0 || hop <= 0 || frame0 < 0)
    return GSS_EINVAL;
  for (int k = 0; k < K; ++k) {
    const uint8_t* a = act_samples + (size_t)k * (size_t)n_samples;
    uint8_t* o = out + (size_t)k * (size_t)n_frames;
    for (int32_t i = 0; i < n_frames; ++i) {
      int64_t c = (frame0 + i - 1) * (int64_t)hop;
      if (c < 0) c = 0;
      if (c > n_samples - 1) c = n_samples - 1;
      o[i] = a[c] != 0;
    }
  }
  return GSS_OK;
}

}  // extern "C"

void gss_profile_begin(gss_ctx* ctx, int which, hipStream_t st) {
  if (!ctx->profile) return;
  if (ctx->ev_used[which] == GSS_PROFILE_SLOTS) (void)drain_profile(ctx, which);   // waits for the oldest launches
  (void)hipEventRecord(ctx->ev_start[which][ctx->ev_used[which]], st);
}

void gss_profile_end(gss_ctx* ctx, int which, hipStream_t st) {
  if (!ctx->profile) return;
  (void)hipEventRecord(ctx->ev_stop[which][ctx->ev_used[which]], st);
  ctx->ev_used[which] += 1;
}

int gss_ensure_scratch(gss_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->scratch_cap) return GSS_OK;
  if (ctx->scratch_fixed) return GSS_ETOOBIG;
  if (hipDeviceSynchronize() != hipSuccess) return GSS_EHIP;
  if (ctx->scratch) {
    (void)hipFree(ctx->scratch);
    ctx->scratch = nullptr;
    ctx->scratch_cap = 0;
  }
  size_t want = gss_align_up(bytes + bytes / 8, (size_t)1 << 20);
  void* p = nullptr;
  if (hipMalloc(&p, want) != hipSuccess) {
    (void)hipGetLastError();
    return GSS_ENOMEM;
  }
  ctx->scratch = p;
  ctx->scratch_cap = want;
  return GSS_OK;
}
