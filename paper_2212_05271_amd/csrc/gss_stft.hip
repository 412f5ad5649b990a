// STFT and inverse STFT around the separation path (arXiv 2212.05271, Section 3: feature extraction and
// iSTFT are among the operations run on the GPU; the paper fixes 513 bins, i.e. a 1024-point transform).
//
// Definition (the paper is silent on window, hop and padding): periodic Hann window of 1024 samples, hop
// 256, the signal zero-padded by 768 samples on both sides, T = ceil(N / 256) + 3 frames; the inverse is
// irfft * window / 1.5 (= sum over the four shifts of the squared window), overlap-added, padding stripped.
//
// A 1024-point real transform is done as a 512-point complex FFT of the even/odd-packed frame plus the
// split step.  The 512-point transform is 8 x 8 x 8: one wavefront per transform, eight values per lane,
// three passes of 8-point butterflies in registers with two exchanges through LDS in between (a radix-2
// transform that lives in LDS is bound by LDS bandwidth: it moves every value through LDS nine times).
// Twiddles come from one table exp(-2 pi i k / 1024), k = 0..512, evaluated in fp64 and rounded once; the
// table is computed on the device by the first call of a context and copied into LDS by every workgroup.
//
// Workgroup order: consecutive workgroup ids go to different XCDs (each with its own L2), so the id is
// remapped such that every XCD walks a contiguous range of frames: neighbouring frames share three quarters
// of their samples, and their 64-byte output runs are neighbours in memory.
#include "gss_internal.h"

namespace {

constexpr int kN = 1024;        // real transform length
constexpr int kH = 512;         // complex transform length
constexpr int kBins = 513;
constexpr int kHop = 256;
constexpr int kPad = kN - kHop;
constexpr int kFftWaves = 8;

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

constexpr int kXcds = 8;

// table[k] = exp(-2 pi i k / 1024), k = 0 .. 512.
__global__ void twiddle_table_kernel(float2* __restrict__ table) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k > kH) return;
  double sn, cs;
  sincospi(-2.0 * (double)k / (double)kN, &sn, &cs);
  table[k] = make_float2((float)cs, (float)sn);
}

// LDS copy of the table, by the whole workgroup (the caller synchronises).
__device__ __forceinline__ void fill_twiddles(float2* tw, const float2* __restrict__ table) {
  for (int k = threadIdx.x; k <= kH; k += blockDim.x) tw[k] = table[k];
}

// Work item of workgroup `id` out of `n` when the grid has kXcds * ceil(n / kXcds) workgroups: XCD x = id % 8
// gets the contiguous items [x * per, (x + 1) * per).  Returns -1 for the padding workgroups.
__device__ __forceinline__ long xcd_contiguous(unsigned id, long n) {
  const long per = (n + kXcds - 1) / kXcds;
  const long w = (long)(id % kXcds) * per + id / kXcds;
  return (id / kXcds < per && w < n) ? w : -1;
}

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// W_1024^idx for 0 <= idx < 1024 from the half table: W^idx = -W^(idx - 512).
__device__ __forceinline__ float2 twiddle(const float2* tw, int idx) {
  const float2 w = tw[idx <= kH ? idx : idx - kH];
  return idx <= kH ? w : make_float2(-w.x, -w.y);
}

// 8-point DFT in registers, natural order in and out: v[k] <- sum_n v[n] exp(-2 pi i n k / 8).
__device__ __forceinline__ void dft8(float2 (&v)[8]) {
  constexpr float kR = 0.70710678118654752440f;
  float2 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a[j] = make_float2(v[j].x + v[j + 4].x, v[j].y + v[j + 4].y);
    b[j] = make_float2(v[j].x - v[j + 4].x, v[j].y - v[j + 4].y);
  }
  // b[j] *= W8^j
  b[1] = make_float2((b[1].x + b[1].y) * kR, (b[1].y - b[1].x) * kR);
  b[2] = make_float2(b[2].y, -b[2].x);
  b[3] = make_float2((b[3].y - b[3].x) * kR, -(b[3].x + b[3].y) * kR);
  // two 4-point DFTs: even outputs from a, odd outputs from b
  auto dft4 = [](const float2 (&c)[4], float2& x0, float2& x1, float2& x2, float2& x3) {
    const float2 e0 = make_float2(c[0].x + c[2].x, c[0].y + c[2].y);
    const float2 e1 = make_float2(c[0].x - c[2].x, c[0].y - c[2].y);
    const float2 o0 = make_float2(c[1].x + c[3].x, c[1].y + c[3].y);
    const float2 d = make_float2(c[1].x - c[3].x, c[1].y - c[3].y);
    const float2 o1 = make_float2(d.y, -d.x);                  // -i (c1 - c3)
    x0 = make_float2(e0.x + o0.x, e0.y + o0.y);
    x2 = make_float2(e0.x - o0.x, e0.y - o0.y);
    x1 = make_float2(e1.x + o1.x, e1.y + o1.y);
    x3 = make_float2(e1.x - o1.x, e1.y - o1.y);
  };
  dft4(a, v[0], v[2], v[4], v[6]);
  dft4(b, v[1], v[3], v[5], v[7]);
}

constexpr int kExStride = 72;                 // float2 per row of the exchange buffer (64 + padding)
constexpr int kExSize = 8 * kExStride;        // >= 512: the buffer also takes the result

// Per-lane constants of the 512-point transform: the twiddles between its passes.
struct FftLane {
  float2 wa[7];     // W_512^(lane * r),          r = 1..7
  float2 wb[7];     // W_64^((lane % 8) * p),     p = 1..7
};
__device__ __forceinline__ void fft_lane_init(FftLane& c, const float2* tw, int lane) {
#pragma unroll
  for (int r = 1; r < 8; ++r) {
    c.wa[r - 1] = twiddle(tw, 2 * lane * r);
    c.wb[r - 1] = twiddle(tw, 16 * (lane & 7) * r);
  }
}

// Forward 512-point complex FFT by one wavefront.  In: v[r] = x[64 r + lane].  Out: the transform in natural
// order in ex[0..511] (visible to the whole wavefront on return).  With n = 64 n1 + n2, k = k1 + 8 k2:
//   pass 1 (lane = n2):            8-point DFT over n1, times W_512^(n2 k1)
//   exchange: rows k1, columns n2 = 8 m1 + m0;   pass 2 (lane = (k1, m0)): DFT over m1, times W_64^(m0 p1)
//   exchange: [k1][p1][m0], 9-float2 pitch;      pass 3 (lane = (k1, p1)): DFT over m0 -> k = k1 + 8 p1 + 64 p0
__device__ __forceinline__ void fft512(float2 (&v)[8], float2* ex, const FftLane& c, int lane) {
  const int hi = lane >> 3, lo = lane & 7;
  dft8(v);
#pragma unroll
  for (int r = 1; r < 8; ++r) v[r] = cmul(v[r], c.wa[r - 1]);
#pragma unroll
  for (int r = 0; r < 8; ++r) ex[r * kExStride + lane] = v[r];
  wave_sync();
#pragma unroll
  for (int m1 = 0; m1 < 8; ++m1) v[m1] = ex[hi * kExStride + 8 * m1 + lo];
  wave_sync();
  dft8(v);
#pragma unroll
  for (int p = 1; p < 8; ++p) v[p] = cmul(v[p], c.wb[p - 1]);
#pragma unroll
  for (int p = 0; p < 8; ++p) ex[hi * kExStride + 9 * p + lo] = v[p];
  wave_sync();
#pragma unroll
  for (int m0 = 0; m0 < 8; ++m0) v[m0] = ex[hi * kExStride + 9 * lo + m0];
  wave_sync();
  dft8(v);
#pragma unroll
  for (int p0 = 0; p0 < 8; ++p0) ex[hi + 8 * lo + 64 * p0] = v[p0];
  wave_sync();
}

// ----------------------------------------------------------------------------------------------
// STFT: one workgroup per (segment, frame); its wavefronts take the channels in turn, eight channels
// at a time are staged in LDS as [bin][channel] and written out as 64-byte runs.
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * kFftWaves) void stft_kernel(const float* __restrict__ x, float2* __restrict__ Y,
                                                             const float2* __restrict__ table, int D, long N, int T,
                                                             long n_items) {
  __shared__ float2 tw[kH + 1];
  __shared__ float2 buf[kFftWaves][kExSize];
  __shared__ float2 stage[kBins][8];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const long item = xcd_contiguous(blockIdx.x, n_items);
  if (item < 0) return;
  const int t = (int)(item % T);
  const int s = (int)(item / T);
  fill_twiddles(tw, table);
  __syncthreads();
  FftLane fc;
  fft_lane_init(fc, tw, lane);
  // periodic Hann window at the lane's samples 2n, 2n + 1, n = 64 m + lane
  float w0[8], w1[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const int i0 = 2 * (lane + 64 * m), i1 = i0 + 1;
    w0[m] = 0.5f - 0.5f * tw[i0 <= kH ? i0 : kN - i0].x;     // cos(2 pi i / 1024) is even around 512
    w1[m] = 0.5f - 0.5f * tw[i1 <= kH ? i1 : kN - i1].x;
  }

  const long start = (long)t * kHop - kPad;      // first sample of the frame (may be negative)
  for (int d0 = 0; d0 < D; d0 += 8) {
    for (int dd = wave; dd < 8; dd += kFftWaves) {
      const int d = d0 + dd;
      if (d < D) {
        const float* __restrict__ xs = x + ((long)s * D + d) * N;
        float2* Z = buf[wave];
        // windowed frame, even/odd packed: z[n] = w[2n] x[2n] + i w[2n+1] x[2n+1]
        float2 v[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const int n = lane + 64 * m;           // 0 .. 511
          const long p0 = start + 2 * n, p1 = p0 + 1;
          const float x0 = (p0 >= 0 && p0 < N) ? xs[p0] : 0.f;
          const float x1 = (p1 >= 0 && p1 < N) ? xs[p1] : 0.f;
          v[m] = make_float2(w0[m] * x0, w1[m] * x1);
        }
        fft512(v, Z, fc, lane);
        // split: X[k] = (Z[k] + conj Z[512-k]) / 2 - i w^k (Z[k] - conj Z[512-k]) / 2, Z[512] = Z[0]
        for (int k = lane; k <= kH; k += 64) {
          const float2 zk = Z[k & (kH - 1)];
          const float2 zc = Z[(kH - k) & (kH - 1)];
          const float2 e = make_float2(0.5f * (zk.x + zc.x), 0.5f * (zk.y - zc.y));
          const float2 o = make_float2(0.5f * (zk.x - zc.x), 0.5f * (zk.y + zc.y));
          const float2 wo = cmul(tw[k], o);      // w^k * o
          stage[k][dd] = make_float2(e.x + wo.y, e.y - wo.x);   // e - i * wo
        }
        wave_sync();                             // Z is reused by this wavefront's next transform
      }
    }
    __syncthreads();
    const int nd = (D - d0) < 8 ? (D - d0) : 8;
    if (nd == 8) {
      for (int i = threadIdx.x; i < kBins * 8; i += blockDim.x) {
        const int k = i >> 3, dd = i & 7;
        Y[(((long)s * kBins + k) * T + t) * D + d0 + dd] = stage[k][dd];
      }
    } else {
      for (int i = threadIdx.x; i < kBins * nd; i += blockDim.x) {
        const int k = i / nd, dd = i % nd;
        Y[(((long)s * kBins + k) * T + t) * D + d0 + dd] = stage[k][dd];
      }
    }
    __syncthreads();
  }
}

// ----------------------------------------------------------------------------------------------
// Inverse STFT, step 1: eight consecutive frames per workgroup (so that the strided reads of X[bin][frame]
// come in 64-byte runs); each wavefront inverts two of them and writes the windowed 1024-sample frames.
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * kFftWaves) void istft_frames_kernel(const float2* __restrict__ X,
                                                                     float* __restrict__ frames,
                                                                     const float2* __restrict__ table, int T) {
  __shared__ float2 tw[kH + 1];
  __shared__ float2 buf[kFftWaves][kExSize];
  __shared__ float2 in[8][kBins + 1];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int groups = (T + 7) / 8;
  const int t0 = (blockIdx.x % groups) * 8;
  const int s = blockIdx.x / groups;
  fill_twiddles(tw, table);
  for (int i = threadIdx.x; i < kBins * 8; i += blockDim.x) {
    const int k = i >> 3, tt = i & 7;
    in[tt][k] = (t0 + tt < T) ? X[((long)s * kBins + k) * T + t0 + tt] : make_float2(0.f, 0.f);
  }
  __syncthreads();
  FftLane fc;
  fft_lane_init(fc, tw, lane);
  for (int tt = wave; tt < 8; tt += kFftWaves) {
    const int t = t0 + tt;
    if (t >= T) break;
    float2* z = buf[wave];
    // pack the half spectrum of a real signal into a 512-point complex one, conjugated so that a forward
    // transform inverts it:  Zc[k] = conj( (X[k] + conj X[512-k]) + i conj(w^k) (X[k] - conj X[512-k]) )
    float2 v[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int k = lane + 64 * m;
      float2 xk = in[tt][k];
      float2 xc = in[tt][kH - k];
      if (k == 0) { xk.y = 0.f; xc.y = 0.f; }    // DC and Nyquist of a real signal are real (as irfft assumes)
      const float2 e = make_float2(xk.x + xc.x, xk.y - xc.y);
      const float2 o = make_float2(xk.x - xc.x, xk.y + xc.y);
      const float2 wc = make_float2(tw[k].x, -tw[k].y);
      const float2 wo = cmul(wc, o);
      v[m] = make_float2(e.x - wo.y, -(e.y + wo.x));          // conj(e + i wo)
    }
    fft512(v, z, fc, lane);
    float* __restrict__ out = frames + ((long)s * T + t) * kN;
    const float scale = 1.0f / (1.5f * (float)kN);            // irfft 1/N, synthesis window / 1.5
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int n = lane + 64 * m;
      const float2 r = z[n];                                   // x[2n] = Re, x[2n+1] = -Im (undo the conjugate)
      const int i0 = 2 * n, i1 = 2 * n + 1;
      const float w0 = 0.5f - 0.5f * tw[i0 <= kH ? i0 : kN - i0].x;
      const float w1 = 0.5f - 0.5f * tw[i1 <= kH ? i1 : kN - i1].x;
      *reinterpret_cast<float2*>(&out[2 * n]) = make_float2(r.x * w0 * scale, -r.y * w1 * scale);
    }
    wave_sync();                                              // z is reused by the next transform
  }
}

// Inverse STFT, step 2: overlap-add.  Sample n (padded position p = n + 768) sums frames p/256 - 3 .. p/256.
__global__ void istft_ola_kernel(const float* __restrict__ frames, float* __restrict__ x, long N, int T) {
  const long n = blockIdx.x * (long)blockDim.x + threadIdx.x;
  const int s = blockIdx.y;
  if (n >= N) return;
  const long p = n + kPad;
  const int th = (int)(p / kHop);
  float acc = 0.f;
#pragma unroll
  for (int q = 3; q >= 0; --q) {                 // fixed order: oldest frame first
    const int t = th - q;
    if (t >= 0 && t < T) acc += frames[((long)s * T + t) * kN + (p - (long)t * kHop)];
  }
  x[(long)s * N + n] = acc;
}

// The context's twiddle table, created on first use; the fill is ordered before the caller's kernels on `st`.
int get_twiddles(gss_ctx* ctx, hipStream_t st, const float2** out) {
  if (!ctx->twiddles) {
    void* p = nullptr;
    if (hipMalloc(&p, (kH + 1) * sizeof(float2)) != hipSuccess) return GSS_ENOMEM;
    hipLaunchKernelGGL(twiddle_table_kernel, dim3((kH + 256) / 256), dim3(256), 0, st, (float2*)p);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess) {
      (void)hipFree(p);
      return GSS_EHIP;
    }
    ctx->twiddles = p;
  }
  *out = (const float2*)ctx->twiddles;
  return GSS_OK;
}

}  // namespace

extern "C" int gss_stft(gss_ctx* ctx, const float* x, int S, int D, int64_t N, int n_fft, int hop,
                        float* Y, int T, void* stream) {
  if (!ctx || !x || !Y || S <= 0 || D <= 0 || N <= 0 || T <= 0) return GSS_EINVAL;
  if (n_fft != kN || hop != kHop) return GSS_EUNSUPPORTED;
  if ((N + hop - 1) / hop + 3 != T) return GSS_EINVAL;
  if ((long)S * T > 0x7ffffff0L) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  const float2* table = nullptr;
  const int rc = get_twiddles(ctx, (hipStream_t)stream, &table);
  if (rc != GSS_OK) return rc;
  const long n_items = (long)S * T;
  const long grid = (n_items + kXcds - 1) / kXcds * kXcds;
  hipLaunchKernelGGL(stft_kernel, dim3((unsigned)grid), dim3(64 * kFftWaves), 0, (hipStream_t)stream, x, (float2*)Y,
                     table, D, (long)N, T, n_items);
  return hipGetLastError() == hipSuccess ? GSS_OK : GSS_EHIP;
}

extern "C" int gss_istft(gss_ctx* ctx, const float* X, int S, int T, int n_fft, int hop,
                         float* x, int64_t N, void* stream) {
  if (!ctx || !X || !x || S <= 0 || T <= 0 || N <= 0) return GSS_EINVAL;
  if (n_fft != kN || hop != kHop) return GSS_EUNSUPPORTED;
  if ((N + hop - 1) / hop + 3 != T) return GSS_EINVAL;
  if (S > 65535) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  const size_t bytes = (size_t)S * T * kN * sizeof(float);
  int rc = gss_ensure_scratch(ctx, bytes);
  if (rc != GSS_OK) return rc;
  float* frames = (float*)ctx->scratch;
  const int groups = (T + 7) / 8;
  if ((long)S * groups > 0x7fffffffL) return GSS_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  const float2* table = nullptr;
  rc = get_twiddles(ctx, st, &table);
  if (rc != GSS_OK) return rc;
  hipLaunchKernelGGL(istft_frames_kernel, dim3((unsigned)(S * groups)), dim3(64 * kFftWaves), 0, st,
                     (const float2*)X, frames, table, T);
  const unsigned nb = (unsigned)((N + 255) / 256);
  hipLaunchKernelGGL(istft_ola_kernel, dim3(nb, (unsigned)S), dim3(256), 0, st, frames, x, (long)N, T);
  return hipGetLastError() == hipSuccess ? GSS_OK : GSS_EHIP;
}
