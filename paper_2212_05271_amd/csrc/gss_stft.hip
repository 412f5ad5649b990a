// STFT and inverse STFT around the separation path (arXiv 2212.05271, Section 3: feature extraction and
// iSTFT are among the operations run on the GPU; the paper fixes 513 bins, i.e. a 1024-point transform).
//
// Definition (the paper is silent on window, hop and padding): periodic Hann window of 1024 samples, hop
// 256, the signal zero-padded by 768 samples on both sides, T = ceil(N / 256) + 3 frames; the inverse is
// irfft * window / 1.5 (= sum over the four shifts of the squared window), overlap-added, padding stripped.
//
// A 1024-point real transform is done as a 512-point complex Stockham radix-2 FFT of the even/odd-packed
// frame in LDS (one wavefront per transform, 64 lanes x 4 butterflies per stage) plus the split step.
// Twiddles come from one table exp(-2 pi i k / 1024), k = 0..512, evaluated in fp64 and rounded once.
#include "gss_internal.h"

namespace {

constexpr int kN = 1024;        // real transform length
constexpr int kH = 512;         // complex transform length
constexpr int kBins = 513;
constexpr int kHop = 256;
constexpr int kPad = kN - kHop;
constexpr int kFftWaves = 4;

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

// tw[k] = exp(-2 pi i k / 1024), k = 0 .. 512, filled by the whole workgroup.
__device__ __forceinline__ void fill_twiddles(float2* tw) {
  for (int k = threadIdx.x; k <= kH; k += blockDim.x) {
    double sn, cs;
    sincospi(-2.0 * (double)k / (double)kN, &sn, &cs);
    tw[k] = make_float2((float)cs, (float)sn);
  }
}

// In-place (ping-pong a <-> b) forward 512-point complex FFT by one wavefront; returns the buffer that
// holds the result.  Stockham autosort, radix 2: at stage Ns (sub-transform size), butterfly j combines
// in[j] and in[j + 256] * w^k, k = j mod Ns, into out[j0] and out[j0 + Ns], j0 = 2 (j - k) + k.
__device__ __forceinline__ float2* fft512(float2* a, float2* b, const float2* tw, int lane) {
  float2* in = a;
  float2* out = b;
#pragma unroll 1
  for (int Ns = 1; Ns < kH; Ns <<= 1) {
    const int tstep = kN / (2 * Ns);          // w = exp(-i pi k / Ns) = tw[k * 1024 / (2 Ns)]
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int j = lane + 64 * m;
      const int k = j & (Ns - 1);
      const int j0 = ((j - k) << 1) + k;
      const float2 u0 = in[j];
      const float2 u1 = cmul(in[j + kH / 2], tw[k * tstep]);
      out[j0] = make_float2(u0.x + u1.x, u0.y + u1.y);
      out[j0 + Ns] = make_float2(u0.x - u1.x, u0.y - u1.y);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float2* t = in; in = out; out = t;
  }
  return in;
}

// ----------------------------------------------------------------------------------------------
// STFT: one workgroup per (segment, frame); its wavefronts take the channels in turn, eight channels
// at a time are staged in LDS as [bin][channel] and written out as 64-byte runs.
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * kFftWaves) void stft_kernel(const float* __restrict__ x, float2* __restrict__ Y,
                                                             int D, long N, int T) {
  __shared__ float2 tw[kH + 1];
  __shared__ float2 buf[kFftWaves][2][kH];
  __shared__ float2 stage[kBins][8];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int t = blockIdx.x % T;
  const int s = blockIdx.x / T;
  fill_twiddles(tw);
  __syncthreads();

  const long start = (long)t * kHop - kPad;      // first sample of the frame (may be negative)
  for (int d0 = 0; d0 < D; d0 += 8) {
    for (int dd = wave; dd < 8; dd += kFftWaves) {
      const int d = d0 + dd;
      if (d < D) {
        const float* __restrict__ xs = x + ((long)s * D + d) * N;
        float2* a = buf[wave][0];
        float2* b = buf[wave][1];
        // windowed frame, even/odd packed: z[n] = w[2n] x[2n] + i w[2n+1] x[2n+1]
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const int n = lane + 64 * m;           // 0 .. 511
          const long p0 = start + 2 * n, p1 = p0 + 1;
          const float x0 = (p0 >= 0 && p0 < N) ? xs[p0] : 0.f;
          const float x1 = (p1 >= 0 && p1 < N) ? xs[p1] : 0.f;
          const int i0 = 2 * n, i1 = 2 * n + 1;
          const float c0 = tw[i0 <= kH ? i0 : kN - i0].x;     // cos(2 pi i / 1024)
          const float c1 = tw[i1 <= kH ? i1 : kN - i1].x;
          a[n] = make_float2((0.5f - 0.5f * c0) * x0, (0.5f - 0.5f * c1) * x1);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const float2* Z = fft512(a, b, tw, lane);
        // split: X[k] = (Z[k] + conj Z[512-k]) / 2 - i w^k (Z[k] - conj Z[512-k]) / 2, Z[512] = Z[0]
        for (int k = lane; k <= kH; k += 64) {
          const float2 zk = Z[k & (kH - 1)];
          const float2 zc = Z[(kH - k) & (kH - 1)];
          const float2 e = make_float2(0.5f * (zk.x + zc.x), 0.5f * (zk.y - zc.y));
          const float2 o = make_float2(0.5f * (zk.x - zc.x), 0.5f * (zk.y + zc.y));
          const float2 wo = cmul(tw[k], o);      // w^k * o
          stage[k][dd] = make_float2(e.x + wo.y, e.y - wo.x);   // e - i * wo
        }
      }
    }
    __syncthreads();
    const int nd = (D - d0) < 8 ? (D - d0) : 8;
    for (int i = threadIdx.x; i < kBins * nd; i += blockDim.x) {
      const int k = i / nd, dd = i % nd;
      Y[(((long)s * kBins + k) * T + t) * D + d0 + dd] = stage[k][dd];
    }
    __syncthreads();
  }
}

// ----------------------------------------------------------------------------------------------
// Inverse STFT, step 1: eight consecutive frames per workgroup (so that the strided reads of X[bin][frame]
// come in 64-byte runs); each wavefront inverts two of them and writes the windowed 1024-sample frames.
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64 * kFftWaves) void istft_frames_kernel(const float2* __restrict__ X,
                                                                     float* __restrict__ frames, int T) {
  __shared__ float2 tw[kH + 1];
  __shared__ float2 buf[kFftWaves][2][kH];
  __shared__ float2 in[8][kBins + 1];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int groups = (T + 7) / 8;
  const int t0 = (blockIdx.x % groups) * 8;
  const int s = blockIdx.x / groups;
  fill_twiddles(tw);
  for (int i = threadIdx.x; i < kBins * 8; i += blockDim.x) {
    const int k = i >> 3, tt = i & 7;
    in[tt][k] = (t0 + tt < T) ? X[((long)s * kBins + k) * T + t0 + tt] : make_float2(0.f, 0.f);
  }
  __syncthreads();
  for (int tt = wave; tt < 8; tt += kFftWaves) {
    const int t = t0 + tt;
    if (t >= T) break;
    float2* a = buf[wave][0];
    float2* b = buf[wave][1];
    // pack the half spectrum of a real signal into a 512-point complex one, conjugated so that a forward
    // transform inverts it:  Zc[k] = conj( (X[k] + conj X[512-k]) + i conj(w^k) (X[k] - conj X[512-k]) )
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
      a[k] = make_float2(e.x - wo.y, -(e.y + wo.x));          // conj(e + i wo)
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float2* z = fft512(a, b, tw, lane);
    float* __restrict__ out = frames + ((long)s * T + t) * kN;
    const float scale = 1.0f / (1.5f * (float)kN);            // irfft 1/N, synthesis window / 1.5
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int n = lane + 64 * m;
      const float2 v = z[n];                                   // x[2n] = Re, x[2n+1] = -Im (undo the conjugate)
      const int i0 = 2 * n, i1 = 2 * n + 1;
      const float w0 = 0.5f - 0.5f * tw[i0 <= kH ? i0 : kN - i0].x;
      const float w1 = 0.5f - 0.5f * tw[i1 <= kH ? i1 : kN - i1].x;
      *reinterpret_cast<float2*>(&out[2 * n]) = make_float2(v.x * w0 * scale, -v.y * w1 * scale);
    }
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

}  // namespace

extern "C" int gss_stft(gss_ctx* ctx, const float* x, int S, int D, int64_t N, int n_fft, int hop,
                        float* Y, int T, void* stream) {
  if (!ctx || !x || !Y || S <= 0 || D <= 0 || N <= 0 || T <= 0) return GSS_EINVAL;
  if (n_fft != kN || hop != kHop) return GSS_EUNSUPPORTED;
  if ((N + hop - 1) / hop + 3 != T) return GSS_EINVAL;
  if ((long)S * T > 0x7fffffffL) return GSS_EUNSUPPORTED;
  if (hipSetDevice(ctx->device) != hipSuccess) return GSS_EHIP;
  hipLaunchKernelGGL(stft_kernel, dim3((unsigned)(S * T)), dim3(64 * kFftWaves), 0, (hipStream_t)stream, x,
                     (float2*)Y, D, (long)N, T);
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
  hipLaunchKernelGGL(istft_frames_kernel, dim3((unsigned)(S * groups)), dim3(64 * kFftWaves), 0, st,
                     (const float2*)X, frames, T);
  const unsigned nb = (unsigned)((N + 255) / 256);
  hipLaunchKernelGGL(istft_ola_kernel, dim3(nb, (unsigned)S), dim3(256), 0, st, frames, x, (long)N, T);
  return hipGetLastError() == hipSuccess ? GSS_OK : GSS_EHIP;
}
